// Fused transform + quantization kernel for 64-wide rows (n2 = 64, n1 = 32 or 64): one wavefront per token, nothing
// shared between tokens after the prologue.  INT4 codes with a step per token, or MXFP4 (template flag).
//
// Same method as the other activation kernels (Eq. (2) left factor, fused as in Sec. 3.3: Z = X~ P2, Y^T = Z^T P1 with Z
// split into fp16 hi + lo, per-token absmax, clip, round, pack), different data movement:
//   * A wave owns a whole token (both 32-column slabs): its rows are fetched with coalesced 16-byte loads (8 whole
//     128-byte rows per instruction), written to a tile of LDS that belongs to this wave alone, and read back as
//     MFMA A operands with 16-byte reads.  No workgroup barrier per token: LDS executes a wave's instructions in
//     order, and the wave waits for its own loads only.  (Fetching the operands straight from global memory in MFMA
//     layout, 32 bytes out of 32 different rows per instruction, was tried first: the vector memory path then needs
//     four times as many cycles per instruction and the rows arrive 2 us later.)
//   * The absmax is a wave reduction, and the codes of a row of X~ (64 channels = 32 bytes) sit in one lane pair
//     (c, 0), (c, 1): one cross-half exchange (v_permlane32_swap) gives each lane 16 contiguous bytes, stored from
//     registers: a wave's store covers 1 KB of consecutive bytes.
//   * Rounding: y / s lands in the top nibble of a 16-bit field through v_cvt_pknorm_i16_f32 (clamp to [-1, 1], times
//     32767, round to nearest): with r = (4096 (u + 0.5) - 0.5) / 32767 the field's top nibble is
//     clamp(rne(u), -8, 7) in two's complement, so clamping, rounding and half of the packing are one fma plus half an
//     instruction per value.  The thresholds between codes move by less than 2e-6 code units (fp32 rounding of the
//     two constants and of the fma), exact ties excepted.
//   * The work of a token is cut by row tiles of X~ (32 rows): a row tile is a K block of the second contraction, so a
//     tile is worked on as soon as its own four loads have arrived, while the other tile's rows are still on their way.
//   * P1 and P2 are requested before the token rows (a CU's vector memory path returns data in request order), staged
//     in LDS once per workgroup and turned into MFMA fragments while the token rows are still on their way from HBM.
#include "fq_internal.h"
#include "fq_device.h"

namespace fq {

// TPW waves (= tokens in flight) per workgroup.  LOOP: persistent workgroups, a wave takes tokens t, t + G, ...
// (G = all waves of the grid) with the next token's rows requested before the current one is worked on.
// MX: MXFP4 output (E2M1 codes, one E8M0 exponent per 32 channels) instead of INT4 codes and a step: the 32 channels of a
// block are the ones a lane pair holds of one slab, so the quantizer needs no wave-wide absmax.
template <int A, int TPW, bool LOOP, bool MX>
__global__ __launch_bounds__(64 * TPW) __attribute__((amdgpu_waves_per_eu(2))) void tq_wave_kernel(const void* __restrict__ aP2, const void* __restrict__ aP1, const void* __restrict__ ax, int64_t ax_stride, int64_t aT,
                    const float* __restrict__ clip, uint8_t* __restrict__ aout_codes, void* __restrict__ aout_scales, int aclip_mode, int amx_tiled) {
    // (plain arguments in the order they are needed, so that the first ones can be delivered in registers at wave start;
    // untyped pointers keep the kernel's name readable in profiler output)
    struct { const _Float16* x; const _Float16* P1; const _Float16* P2; uint8_t* out_codes; void* out_scales; int64_t x_stride, T; int clip_mode, mx_tiled; } p =
        {static_cast<const _Float16*>(ax), static_cast<const _Float16*>(aP1), static_cast<const _Float16*>(aP2), aout_codes,
         aout_scales, ax_stride, aT, aclip_mode, amx_tiled};
    constexpr int N1 = 32 * A, N2 = 64, KB1 = 2 * A, KB2 = 4, NT = 64 * TPW;
    constexpr int CH2 = N2 * N2 / 8, CH1 = N1 * N1 / 8, CH = CH1 + CH2;   // 16-byte chunks of P2, P1
    constexpr int NLD = (CH + NT - 1) / NT;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    _Float16* P2flat = reinterpret_cast<_Float16*>(smem);
    _Float16* P1flat = P2flat + N2 * N2;
    constexpr int TILE_BYTES = N1 * N2 * 2;          // one token, rows unpadded (the loads write whole 1 KB runs)

    const int tid = threadIdx.x;
    const int l = tid & 63, c = l & 31, h = l >> 5;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    unsigned char* tile = smem + CH * 16 + wv * TILE_BYTES;
    const int64_t G = (int64_t)gridDim.x * TPW;
    int64_t t = (int64_t)blockIdx.x * TPW + wv;
    if (t >= p.T) t = p.T - 1;                       // spare waves of the last workgroup redo token T - 1: same bytes stored twice

    // ---- requests: the transforms first, then this wave's first token
    u32x4 pv[NLD];
#pragma unroll
    for (int k = 0; k < NLD; ++k) {
        int idx = tid + k * NT;
        if (idx >= CH) idx = CH - 1;
        const u32x4* src = idx < CH2 ? reinterpret_cast<const u32x4*>(p.P2) + idx : reinterpret_cast<const u32x4*>(p.P1) + (idx - CH2);
        pv[k] = *src;
    }
    // Token rows: load k brings rows 8 k .. 8 k + 7 (lane i: 16 bytes; every byte of the token is read once, whole
    // 128-byte lines per 8 lanes), and is written to LDS at tile + 1024 k + 16 i.  Slot j of row r holds the row's chunk
    // j ^ ((r >> 1) & 7): with that swizzle the 16-byte operand reads of 32 consecutive rows (same chunk) spread over all
    // banks although the pitch is a multiple of the bank width.
    constexpr int NROW = N1 / 8;
    const int ld_ofs = (l >> 3) * (N2 * 2) + 16 * ((l & 7) ^ ((l >> 4) & 3));   // rows 8 k + l / 8: (r >> 1) & 7 = 4 (k & 1) + (l >> 4)
    auto issue = [&](int64_t tok, u32x4 (&pre)[NROW], int It) {   // row tile It, or all of them (It < 0)
        const unsigned char* row = reinterpret_cast<const unsigned char*>(p.x + tok * p.x_stride);
#pragma unroll
        for (int k = (It < 0 ? 0 : 4 * It); k < (It < 0 ? NROW : 4 * It + 4); ++k)
            pre[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(row + k * (8 * N2 * 2) + (ld_ofs ^ (64 * (k & 1)))));
    };
    // (row tile It = loads 4 It .. 4 It + 3 = 4 KB of the tile)
    auto commit = [&](const u32x4 (&pre)[NROW], int It) {
#pragma unroll
        for (int k = 4 * It; k < 4 * It + 4; ++k) *reinterpret_cast<u32x4*>(tile + k * 1024 + 16 * l) = pre[k];
    };
    // lane (c, h), row tile It, K block kb: X~[32 It + c][16 kb + 8 h .. + 7] = chunk 2 kb + h of row 32 It + c
    const int rd_ofs = c * (N2 * 2);
    const int rd_swz = (c >> 1) & 7;
    auto fetch = [&](u32x4 (&a)[KB2], int It) {
#pragma unroll
        for (int kb = 0; kb < KB2; ++kb)
            a[kb] = *reinterpret_cast<const u32x4*>(tile + It * (32 * N2 * 2) + rd_ofs + 16 * ((2 * kb + h) ^ rd_swz));
    };
    u32x4 pre[NROW];
    // A CU's vector memory path takes requests and returns data in order, whatever wave they come from: the barrier
    // puts every wave's share of P1 / P2 (L2) in front of every wave's token rows (HBM).  Without it the last wave's
    // share queues behind the other waves' rows and the fragments are ready no sooner than the rows.
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    issue(t, pre, -1);
    __builtin_amdgcn_sched_barrier(0);

    // ---- transforms -> LDS -> fragments (while the token rows are in flight)
#pragma unroll
    for (int k = 0; k < NLD; ++k) {
        const int idx = tid + k * NT;
        if (CH % NT == 0 || idx < CH) reinterpret_cast<u32x4*>(smem)[idx] = pv[k];   // (the compiler's wait covers the older P loads only)
    }
    __syncthreads();
    // B operand of the first contraction: lane (c, h) holds P2[16 kb + 8 h + s][32 q + c], s = 0..7
    half8 p2f[2][KB2];
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int kb = 0; kb < KB2; ++kb) p2f[q][kb] = lds_column8(P2flat, N2, 16 * kb + 8 * h, 4, 32 * q + (c & 16), l & 15);
    // B operand of the second contraction, gathered with the K permutation of the accumulator layout that feeds it:
    // K block kk, slot s, half-wave h  <->  i = 32 (kk / 2) + 8 (2 (kk % 2) + s / 4) + 4 h + s % 4
    half8 p1f[A][KB1];
#pragma unroll
    for (int It = 0; It < A; ++It)
#pragma unroll
        for (int kk = 0; kk < KB1; ++kk)
            p1f[It][kk] = lds_column8(P1flat, N1, 32 * (kk >> 1) + 16 * (kk & 1) + 4 * h, 8, 32 * It + (c & 16), l & 15);

    // ---- one token.  The work is cut by row tiles of X~ (32 rows = 4 KB = half of a 64 x 64 token): both contractions of
    // a row tile need nothing of the other one (it is a K block of the second contraction), so a tile is worked on as soon
    // as its own rows have arrived.  The schedule of a tile is written out: the wave has nobody to hide its own latencies
    // behind but itself (and one other wave of its SIMD), so the vector-ALU work of one slab runs in the shadow of the
    // other slab's MFMAs.
    //   H1  Z0 = X~[tile] P2[:, slab 0]                       (MFMA)
    //   H2  Z1 = X~[tile] P2[:, slab 1]                       (MFMA)   |  split Z0 into hi + lo        (VALU)
    //   H3  Y^T[slab 0] += Z0^T P1[tile rows], hi and lo     (MFMA)   |  split Z1                      (VALU)
    //   H4  Y^T[slab 1] += Z1^T P1[tile rows]                (MFMA)   |  last tile: absmax over slab 0 (VALU)
    // then absmax over slab 1, step, round, pack, store.
    f32x16 acc2[2][A];
    float m;
    auto absmax_part = [&](int q, int u) {   // half of slab q's accumulators
#pragma unroll
        for (int j = 0; j < 8 * A; j += 2) {
            const int e = u * (8 * A) + j;
            m = __builtin_fmaxf(__builtin_fmaxf(m, __builtin_fabsf(acc2[q][e / 16][e % 16])), __builtin_fabsf(acc2[q][e / 16][e % 16 + 1]));
        }
    };
    auto clear = [&]() {
        m = 0.0f;
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int I2 = 0; I2 < A; ++I2)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc2[q][I2][r] = 0.0f;
    };
    auto row_tile = [&](int It, const u32x4 (&xr)[KB2]) {
        f32x16 acc1[2];
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc1[q][r] = 0.0f;
        half8 zh[2][2], zl[2][2];
        auto first = [&](int q, int kb) {
            acc1[q] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, xr[kb]), p2f[q][kb], acc1[q], 0, 0, 0);
        };
        auto second = [&](int q, int kq) {   // K block kk = 2 It + kq: 16 rows of X~
#pragma unroll
            for (int I2 = 0; I2 < A; ++I2) acc2[q][I2] = __builtin_amdgcn_mfma_f32_32x32x16_f16(zh[q][kq], p1f[I2][2 * It + kq], acc2[q][I2], 0, 0, 0);
#pragma unroll
            for (int I2 = 0; I2 < A; ++I2) acc2[q][I2] = __builtin_amdgcn_mfma_f32_32x32x16_f16(zl[q][kq], p1f[I2][2 * It + kq], acc2[q][I2], 0, 0, 0);
        };
        // H1
#pragma unroll
        for (int kb = 0; kb < KB2; ++kb) first(0, kb);
        __builtin_amdgcn_sched_barrier(0);
        // H2
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            first(1, 2 * g);
            first(1, 2 * g + 1);
            split_hi_lo(acc1[0], 8 * g, zh[0][g], zl[0][g]);
            __builtin_amdgcn_sched_barrier(0);
        }
        // H3
#pragma unroll
        for (int kq = 0; kq < 2; ++kq) {
            second(0, kq);
            split_hi_lo(acc1[1], 8 * kq, zh[1][kq], zl[1][kq]);
            __builtin_amdgcn_sched_barrier(0);
        }
        // H4
#pragma unroll
        for (int kq = 0; kq < 2; ++kq) {
            second(1, kq);
            if (!MX && It == A - 1) absmax_part(0, kq);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // lane pair exchange of the packed codes: W[q][mm] holds, for slab q, the lane's 4 + 4 channels of groups g = 2 mm
    // and 2 mm + 1 (2 + 2 bytes); afterwards lane (c, h) holds slab q = h of both lanes, 16 consecutive bytes of the row
    auto store_codes = [&](uint8_t* dst, const uint32_t (&W)[2][2]) {
        u32x4 o;
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) {
            const auto sw = __builtin_amdgcn_permlane32_swap(W[0][mm], W[1][mm], false, false);
            const uint32_t P = sw[0], Q = sw[1];                        // half-wave 0's, half-wave 1's
            o[2 * mm] = __builtin_amdgcn_perm(Q, P, 0x05040100u);       // group g = 2 mm: 2 bytes of P, 2 bytes of Q
            o[2 * mm + 1] = __builtin_amdgcn_perm(Q, P, 0x07060302u);   // group g = 2 mm + 1
        }
        __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(dst));
    };
    auto finish = [&](int64_t tok) {
        const float clipv = clip[p.clip_mode ? tok : 0];   // wave-uniform address: a scalar load
        // Lane (c, h) holds, of row ip = 32 It + c of X~, the channels 32 q + 8 g + 4 h + k in acc2[q][It][4 g + k].
        uint8_t* out_row = p.out_codes + tok * (int64_t)(N1 * N2 / 2) + c * (N2 / 2) + 16 * h;
        if constexpr (MX) {
            // Block (ip, q) = the 32 values of the lane pair (c, 0), (c, 1) in acc2[q][It]: exponent floor(log2(alpha max)) - 2
            // (0 for an all-zero block), elements converted with the stored exponent (the conversion reads the exponent
            // field of its scale operand only, and field 0 means 2^-127).
            uint8_t* exps = reinterpret_cast<uint8_t*>(p.out_scales);
#pragma unroll
            for (int It = 0; It < A; ++It) {
                uint32_t W[2][2], e2 = 0;
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    float bm = 0.0f;
#pragma unroll
                    for (int r = 0; r < 16; r += 2) bm = __builtin_fmaxf(__builtin_fmaxf(bm, __builtin_fabsf(acc2[q][It][r])), __builtin_fabsf(acc2[q][It][r + 1]));
                    const auto sw = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(uint32_t, bm), __builtin_bit_cast(uint32_t, bm), false, false);
                    bm = __builtin_fmaxf(__builtin_bit_cast(float, (uint32_t)sw[0]), __builtin_bit_cast(float, (uint32_t)sw[1])) * clipv;
                    const uint32_t be = (__builtin_bit_cast(uint32_t, bm) >> 23) & 0xffu;
                    const uint32_t e = be > 2 ? be - 2 : 0;
                    const float scale = __builtin_bit_cast(float, e << 23);
                    e2 |= e << (8 * q);
#pragma unroll
                    for (int mm = 0; mm < 2; ++mm) {
                        // byte j: channels 2 (j % 2), 2 (j % 2) + 1 of group g = 2 mm + j / 2 (the byte index must be a literal)
                        const f32x16& y = acc2[q][It];
                        uint32_t pk = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(0u, y[8 * mm], y[8 * mm + 1], scale, 0);
                        pk = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(pk, y[8 * mm + 2], y[8 * mm + 3], scale, 1);
                        pk = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(pk, y[8 * mm + 4], y[8 * mm + 5], scale, 2);
                        pk = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(pk, y[8 * mm + 6], y[8 * mm + 7], scale, 3);
                        W[q][mm] = pk;
                    }
                }
                store_codes(out_row + It * (32 * N2 / 2), W);
                // exponents: two bytes per row of X~ (index 2 ip + q)
                const int ip = 32 * It + c;
                if (!p.mx_tiled) {
                    if (h == 0) *reinterpret_cast<uint16_t*>(exps + tok * (int64_t)(2 * N1) + 2 * ip) = (uint16_t)e2;
                } else {
                    // tile order of the MXFP4 product: tokens in tiles of 128; per tile and K iteration j (256 channels = 4
                    // rows of X~ = 8 exponents) the 128 tokens' 8 bytes are contiguous.  The four lanes of a quad hold the
                    // four rows of one iteration: lane 0 of the quad gathers them and stores 8 bytes.
                    const uint32_t a1 = __builtin_amdgcn_mov_dpp((int)e2, 0x55, 0xF, 0xF, true);   // quad lane 1's
                    const uint32_t a2 = __builtin_amdgcn_mov_dpp((int)e2, 0xAA, 0xF, 0xF, true);
                    const uint32_t a3 = __builtin_amdgcn_mov_dpp((int)e2, 0xFF, 0xF, 0xF, true);
                    constexpr int KI = N1 * N2 / 256;
                    if (h == 0 && (c & 3) == 0) {
                        uint2 v;
                        v.x = e2 | (a1 << 16);
                        v.y = a2 | (a3 << 16);
                        reinterpret_cast<uint2*>(exps)[((tok >> 7) * KI + (ip >> 2)) * 128 + (tok & 127)] = v;
                    }
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < 2; ++u) absmax_part(1, u);
            m = wave_max(m);
            // ---- step = alpha * max / 7, rounded to fp16; the rounded step divides
            const _Float16 sh = (_Float16)(clipv * m * 0.142857149f);
            const float s = (float)sh;
            const float inv = (s > 0.0f && s <= 65504.0f) ? __builtin_amdgcn_rcpf(s) : 0.0f;   // 1 ulp: < 1e-6 code units
            const float kmul = inv * (4096.0f / 32767.0f);
            constexpr float kadd = 2047.5f / 32767.0f;
            // ---- round, clamp, pack: eight values (g = 2 m, 2 m + 1) become one dword of nibbles
#pragma unroll
            for (int It = 0; It < A; ++It) {
                uint32_t W[2][2];
#pragma unroll
                for (int q = 0; q < 2; ++q)
#pragma unroll
                    for (int mm = 0; mm < 2; ++mm) {
                        uint32_t D[4];
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            const float r0 = __builtin_fmaf(acc2[q][It][8 * mm + k], kmul, kadd);
                            const float r1 = __builtin_fmaf(acc2[q][It][8 * mm + 4 + k], kmul, kadd);
                            D[k] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pknorm_i16(r0, r1));
                        }
                        // bytes 1 and 3 of D[k] carry nibbles k and k + 4 on top: even nibbles -> E, odd ones -> F
                        const uint32_t E = __builtin_amdgcn_perm(D[2], D[0], 0x07030501u);
                        const uint32_t F = __builtin_amdgcn_perm(D[3], D[1], 0x07030501u);
                        W[q][mm] = (F & 0xF0F0F0F0u) | ((E >> 4) & 0x0F0F0F0Fu);
                    }
                store_codes(out_row + It * (32 * N2 / 2), W);
            }
            reinterpret_cast<_Float16*>(p.out_scales)[tok] = sh;   // every lane writes the same two bytes: cheaper than a branch around the store
        }
    };

    __builtin_amdgcn_sched_barrier(0);   // the fragment reads are issued before anything waits for the token rows
    // The tile belongs to this wave alone and LDS executes a wave's instructions in order: no barrier between writing
    // the rows and reading them back as operands, nor before the next token's rows overwrite them.
    u32x4 xr[KB2];
    if constexpr (!LOOP) {
        clear();
#pragma unroll
        for (int It = 0; It < A; ++It) {
            commit(pre, It);
            fetch(xr, It);
            __builtin_amdgcn_sched_barrier(0);
            row_tile(It, xr);
        }
        finish(t);
    } else {
        // Past the end a wave re-reads the last token's rows: an unconditional request keeps the compiler's count of
        // outstanding loads exact, so the wait before a row tile covers its rows only.
        while (true) {
            const int64_t tn = t + G;
            const int64_t tr = tn < p.T ? tn : p.T - 1;
            clear();
#pragma unroll
            for (int It = 0; It < A; ++It) {
                commit(pre, It);
                fetch(xr, It);
                issue(tr, pre, It);
                __builtin_amdgcn_sched_barrier(0);
                row_tile(It, xr);
            }
            finish(t);
            t = tn;
            if (t >= p.T) break;
        }
    }
}

// ------------------------------------------------------------------------------------
// Left factor only, 128-wide rows (the online part of P_o: heads x head_dim with P2 = I; n1 = 32 or 64): Y = P1^T X~,
// one wavefront per token, loop-free.  There is no first contraction and no hi / lo split: the second contraction's
// operand is X~ itself (exact fp16), gathered from the wave's tile with transposing reads (rows i = K, columns = the
// slab's 32 channels), so the tile keeps plain rows at a padded pitch instead of the swizzle.  A token row is
// contiguous in memory, so load k is simply bytes 1024 k .. of the token (4 rows of X~).  Row tiles as above: the
// K blocks of a 32-row tile are multiplied as soon as its eight loads have arrived.
template <int A, int TPW>
__global__ __launch_bounds__(64 * TPW) __attribute__((amdgpu_waves_per_eu(2))) void po_wave_kernel(const void* __restrict__ aP1, const void* __restrict__ ax, int64_t x_stride, int64_t T,
                    const float* __restrict__ clip, uint8_t* __restrict__ out_codes, void* __restrict__ out_scales, int clip_mode) {
    constexpr int N1 = 32 * A, N2 = 128, KB1 = 2 * A, NT = 64 * TPW, NQ = 4;
    constexpr int CH1 = N1 * N1 / 8;                  // 16-byte chunks of P1
    constexpr int NLD = (CH1 + NT - 1) / NT;
    constexpr int PITCH = N2 + 8;                     // halves per tile row: 16 bytes of padding keep the transposing reads off one bank group
    constexpr int TILE_BYTES = N1 * PITCH * 2;
    constexpr int LPT = 8, NROW = A * LPT;            // loads of 1 KB per row tile, per token

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    _Float16* P1flat = reinterpret_cast<_Float16*>(smem);
    const int tid = threadIdx.x;
    const int l = tid & 63, c = l & 31, h = l >> 5;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    _Float16* tile = reinterpret_cast<_Float16*>(smem + CH1 * 16 + wv * TILE_BYTES);
    int64_t t = (int64_t)blockIdx.x * TPW + wv;
    if (t >= T) t = T - 1;                            // spare waves of the last workgroup redo token T - 1: same bytes stored twice

    u32x4 pv[NLD];
#pragma unroll
    for (int k = 0; k < NLD; ++k) {
        const int idx = tid + k * NT;
        pv[k] = reinterpret_cast<const u32x4*>(aP1)[idx < CH1 ? idx : CH1 - 1];
    }
    // P1 (L2) in front of every wave's token rows (HBM) in the CU's request queue, as in the kernel above
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    u32x4 pre[NROW];
    {
        const unsigned char* row = reinterpret_cast<const unsigned char*>(static_cast<const _Float16*>(ax) + t * x_stride);
#pragma unroll
        for (int k = 0; k < NROW; ++k) pre[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(row + k * 1024 + 16 * l));
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < NLD; ++k) {
        const int idx = tid + k * NT;
        if (CH1 % NT == 0 || idx < CH1) reinterpret_cast<u32x4*>(smem)[idx] = pv[k];
    }
    __syncthreads();
    // B operand, gathered with the K permutation of the operand layout that feeds it (see the kernel above)
    half8 p1f[A][KB1];
#pragma unroll
    for (int It = 0; It < A; ++It)
#pragma unroll
        for (int kk = 0; kk < KB1; ++kk)
            p1f[It][kk] = lds_column8(P1flat, N1, 32 * (kk >> 1) + 16 * (kk & 1) + 4 * h, 8, 32 * It + (c & 16), l & 15);
    __builtin_amdgcn_sched_barrier(0);

    const float clipv = clip[clip_mode ? t : 0];
    f32x16 acc2[NQ][A];
#pragma unroll
    for (int q = 0; q < NQ; ++q)
#pragma unroll
        for (int It = 0; It < A; ++It)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc2[q][It][r] = 0.0f;
#pragma unroll
    for (int Ir = 0; Ir < A; ++Ir) {
        // rows 32 Ir .. 32 Ir + 31 of X~: load k covers rows 4 k .. 4 k + 3 (16 lanes per row)
#pragma unroll
        for (int k = LPT * Ir; k < LPT * Ir + LPT; ++k)
            *reinterpret_cast<u32x4*>(tile + (4 * k + (l >> 4)) * PITCH + 8 * (l & 15)) = pre[k];
        // (the tile is this wave's alone and LDS executes a wave's instructions in order; the fences only keep the compiler
        // from moving the transposing reads above the writes)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int kq = 0; kq < 2; ++kq) {
            const int kk = 2 * Ir + kq;
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const half8 z = lds_column8(tile, PITCH, 32 * (kk >> 1) + 16 * (kk & 1) + 4 * h, 8, 32 * q + (c & 16), l & 15);
#pragma unroll
                for (int It = 0; It < A; ++It) acc2[q][It] = __builtin_amdgcn_mfma_f32_32x32x16_f16(z, p1f[It][kk], acc2[q][It], 0, 0, 0);
            }
        }
    }
    // ---- absmax, step, round, pack, store: as in the kernel above, two slab pairs per row of X~
    float m = 0.0f;
#pragma unroll
    for (int q = 0; q < NQ; ++q)
#pragma unroll
        for (int It = 0; It < A; ++It)
#pragma unroll
            for (int r = 0; r < 16; r += 2) m = __builtin_fmaxf(__builtin_fmaxf(m, __builtin_fabsf(acc2[q][It][r])), __builtin_fabsf(acc2[q][It][r + 1]));
    m = wave_max(m);
    const _Float16 sh = (_Float16)(clipv * m * 0.142857149f);
    const float s = (float)sh;
    const float inv = (s > 0.0f && s <= 65504.0f) ? __builtin_amdgcn_rcpf(s) : 0.0f;
    const float kmul = inv * (4096.0f / 32767.0f);
    constexpr float kadd = 2047.5f / 32767.0f;
    uint8_t* out_row = out_codes + t * (int64_t)(N1 * N2 / 2) + c * (N2 / 2) + 16 * h;
#pragma unroll
    for (int It = 0; It < A; ++It)
#pragma unroll
        for (int qp = 0; qp < NQ / 2; ++qp) {
            u32x4 o;
#pragma unroll
            for (int mm = 0; mm < 2; ++mm) {
                uint32_t W[2];
#pragma unroll
                for (int qq = 0; qq < 2; ++qq) {
                    const f32x16& y = acc2[2 * qp + qq][It];
                    uint32_t D[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        D[k] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pknorm_i16(__builtin_fmaf(y[8 * mm + k], kmul, kadd), __builtin_fmaf(y[8 * mm + 4 + k], kmul, kadd)));
                    const uint32_t E = __builtin_amdgcn_perm(D[2], D[0], 0x07030501u);
                    const uint32_t F = __builtin_amdgcn_perm(D[3], D[1], 0x07030501u);
                    W[qq] = (F & 0xF0F0F0F0u) | ((E >> 4) & 0x0F0F0F0Fu);
                }
                const auto sw = __builtin_amdgcn_permlane32_swap(W[0], W[1], false, false);
                o[2 * mm] = __builtin_amdgcn_perm(sw[1], sw[0], 0x05040100u);
                o[2 * mm + 1] = __builtin_amdgcn_perm(sw[1], sw[0], 0x07060302u);
            }
            __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(out_row + It * (32 * N2 / 2) + 32 * qp));
        }
    static_cast<_Float16*>(out_scales)[t] = sh;
}

bool po_wave_applicable(const TqDev& d) {
    if (d.P2 || !d.P1 || d.n2 != 128 || (d.n1 != 32 && d.n1 != 64) || !d.vec8 || !d.out_vec16) return false;
    if (reinterpret_cast<uintptr_t>(d.P1) & 15) return false;
    return d.T >= 1 && d.T <= 0x7fffffff;
}

hipError_t po_wave_launch(const TqDev& d, hipStream_t stream) {
    constexpr int TPW = 4;
    using Fn = void (*)(const void*, const void*, int64_t, int64_t, const float*, uint8_t*, void*, int);
    const bool two = d.n1 == 64;
    Fn fn = two ? &po_wave_kernel<2, TPW> : &po_wave_kernel<1, TPW>;
    const int lds = d.n1 * d.n1 * 2 + TPW * d.n1 * (128 + 8) * 2;
    static OccCache occ_cache[2];   // the first call also raises the kernel's LDS limit
    int occ = 0;
    hipError_t e = kernel_occupancy(reinterpret_cast<const void*>(fn), 64 * TPW, lds, occ_cache[two], occ);
    if (e != hipSuccess) return e;
    return launch(fn, dim3((unsigned)((d.T + TPW - 1) / TPW)), dim3(64 * TPW), lds, stream, d.P1, d.x, d.x_stride, d.T, d.clip, d.out_codes, d.out_scales, d.clip_mode);
}

// ------------------------------------------------------------------------------------
bool tq_wave_applicable(const TqDev& d) {
    if (d.n2 != 64 || (d.n1 != 32 && d.n1 != 64) || !d.P1 || !d.P2 || !d.vec8 || !d.out_vec16) return false;
    if ((reinterpret_cast<uintptr_t>(d.P1) | reinterpret_cast<uintptr_t>(d.P2)) & 15) return false;
    return d.T >= 1 && d.T <= 0x7fffffff;
}

using WaveFn = void (*)(const void*, const void*, const void*, int64_t, int64_t, const float*, uint8_t*, void*, int, int);
template <int TPW, bool MX>
static WaveFn wave_fn(int A, bool loop) {
    if (A == 1) return loop ? &tq_wave_kernel<1, TPW, true, MX> : &tq_wave_kernel<1, TPW, false, MX>;
    return loop ? &tq_wave_kernel<2, TPW, true, MX> : &tq_wave_kernel<2, TPW, false, MX>;
}

// tpw: 2, 4 or 8 waves per workgroup; loop: persistent workgroups (grid = as many as are resident), else one token per
// wave; mx: MXFP4 output (d.mx_tiled: exponents in the product's tile order)
hipError_t tq_wave_launch(const TqDev& d, hipStream_t stream, int tpw, bool loop, bool mx) {
    const int A = d.n1 / 32;
    if (tpw != 2 && tpw != 4) tpw = 8;
    WaveFn fn = mx ? (tpw == 2 ? wave_fn<2, true>(A, loop) : tpw == 4 ? wave_fn<4, true>(A, loop) : wave_fn<8, true>(A, loop))
                   : (tpw == 2 ? wave_fn<2, false>(A, loop) : tpw == 4 ? wave_fn<4, false>(A, loop) : wave_fn<8, false>(A, loop));
    const int lds = (64 * 64 + d.n1 * d.n1) * 2 + tpw * d.n1 * 64 * 2;   // P2, P1, one tile per wave
    static OccCache occ_cache[2][2][3][2];   // per variant and device; the first call also raises the kernel's LDS limit
    int occ = 0;
    {
        hipError_t e = kernel_occupancy(reinterpret_cast<const void*>(fn), 64 * tpw, lds, occ_cache[mx][A - 1][tpw == 2 ? 0 : tpw == 4 ? 1 : 2][loop], occ);
        if (e != hipSuccess) return e;
    }
    int64_t grid = (d.T + tpw - 1) / tpw;
    if (loop) {
        // every wave gets the same number of tokens (+-1)
        const int64_t resident = (int64_t)cu_count() * occ;
        const int64_t rounds = (grid + resident - 1) / resident;
        grid = (grid + rounds - 1) / rounds;
    }
    return launch(fn, dim3((unsigned)grid), dim3(64 * tpw), lds, stream, d.P2, d.P1, d.x, d.x_stride, d.T, d.clip, d.out_codes, d.out_scales, d.clip_mode, d.mx_tiled);
}

}  // namespace fq
