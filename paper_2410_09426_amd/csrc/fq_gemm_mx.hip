// Product of two MXFP4 factors on gfx950's scaled FP4 MFMA: out[t, o] = fp16( sum_k x^[t, k] w^[o, k] ), the low-bit
// matrix multiplication of Sec. 3.2 for the data type the paper's "Limitations" name next.  x^ and w^ are the
// de-quantized outputs of flatquant_transform_mxfp4_tiled (activations [T, n/2] codes + n/32 exponents per token in
// tile order, weights likewise): E2M1 elements times one power of two per block of 32 consecutive channels.
//
// v_mfma_scale_f32_32x32x64_f8f6f4 with both formats FP4 takes, per lane, 32 consecutive K elements (16 bytes of
// packed nibbles: lane (c, h) <-> row c, K half h) and one E8M0 exponent for exactly those 32 elements, so the stored
// layout is the operand layout: no unpacking, no widening, the block scales are applied inside the MFMA (measured on
// the device: the result equals the fp64 sum for random operands whose partial sums fit fp32).
//
// Workgroup and data movement as in the INT4 product (fq_gemm.hip): 4 waves, C tile 128 tokens x 128 output channels,
// 64 x 64 per wave with the weights as the MFMA's first operand; K advances by 256 codes per iteration through
// double-buffered LDS tiles filled by global-to-LDS loads (unpadded rows, 16-byte chunks swizzled), one barrier per
// iteration.  The exponents (8 bytes per row and iteration, stored in tile order) travel the same way.
// (A ring of four 128-code stages with three in flight measured slower: 64-byte row pieces multiply the number of
// L2 requests.)
#include "fq_internal.h"

namespace fq {

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int XT = 128;               // tile edge, tokens and output channels
constexpr int XKB = 128;              // packed bytes of K per row and iteration (256 codes, 8 blocks)
constexpr int X_NT = 256;
constexpr int X_TILE_BYTES = XT * XKB;
constexpr int X_EXP_BYTES = 2 * XT * 8;         // exponents of both tiles for one iteration: 8 bytes per row
constexpr int X_LDS_BYTES = 4 * X_TILE_BYTES + 2 * X_EXP_BYTES;   // A and B, two buffers each (the output tile reuses them), + exponents

struct MxGemmDev {
    const uint8_t* xc;
    const uint8_t* xe;
    const uint8_t* wc;
    const uint8_t* we;
    _Float16* out;
    int64_t T;
    int64_t out_stride;
    int m, n;
};

__global__ __launch_bounds__(X_NT) __attribute__((amdgpu_waves_per_eu(2))) void mxfp4_gemm_kernel(MxGemmDev p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x;
    const int l = tid & 63, c = l & 31, h = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w & 1, wn = w >> 1;
    const int64_t t0 = (int64_t)blockIdx.x * XT;
    const int o0 = blockIdx.y * XT;
    const int64_t kbytes = p.n / 2;
    const int nk = p.n / (2 * XKB);

    // code tiles: one instruction fills 8 rows of 128 bytes; wave w owns rows 32 w .. 32 w + 31 of both tiles.  LDS slot
    // j of row r holds the row's chunk j ^ ((r >> 1) & 7).  Rows past the end re-read the last row.
    constexpr int NLD = 4;
    const unsigned char* asrc[NLD];
    const unsigned char* bsrc[NLD];
#pragma unroll
    for (int k = 0; k < NLD; ++k) {
        const int row = 8 * (4 * w + k) + (l >> 3), ch = (l & 7) ^ ((row >> 1) & 7);
        int64_t tr = t0 + row;
        if (tr >= p.T) tr = p.T - 1;
        int orow = o0 + row;
        if (orow >= p.m) orow = p.m - 1;
        asrc[k] = p.xc + tr * kbytes + 16 * ch;
        bsrc[k] = p.wc + (int64_t)orow * kbytes + 16 * ch;
    }
    typedef const __attribute__((address_space(1))) void* gptr;
    typedef __attribute__((address_space(3))) void* lptr;
    auto issue = [&](int it, int buf) {   // past the last tile the last one is re-read (nobody uses it)
        const int itc = it < nk ? it : nk - 1;
        unsigned char* A = smem + buf * X_TILE_BYTES + w * (32 * XKB);
        unsigned char* B = smem + (2 + buf) * X_TILE_BYTES + w * (32 * XKB);
#pragma unroll
        for (int k = 0; k < NLD; ++k) {
            __builtin_amdgcn_global_load_lds((gptr)(asrc[k] + (int64_t)itc * XKB), (lptr)(A + k * 8 * XKB), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((gptr)(bsrc[k] + (int64_t)itc * XKB), (lptr)(B + k * 8 * XKB), 16, 0, 0);
        }
    };
    auto tile_ready = [&]() {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    };

    // Exponents: 8 bytes per row and iteration, stored in tile order (rows in tiles of 128; per tile and iteration the
    // 128 rows' 8 bytes are contiguous), so one iteration's exponents of a tile are 1 KB in one piece: one global-to-LDS
    // instruction per operand, issued with the code tiles (wave 0: tokens, wave 1: channels).  Measured on the way: with
    // row-major exponents fetched into registers (8 bytes per lane, row and iteration: four times as many cache lines
    // touched per iteration as the code tiles) the exponents took 45 % of the kernel's time; fetched through LDS 32
    // bytes per row at a time, still 25 %.
    const int64_t tile_e = (int64_t)nk * 1024;   // bytes of exponents per tile of 128 rows
    const unsigned char* xsrc = (w == 0 ? p.xe + (int64_t)blockIdx.x * tile_e : p.we + (int64_t)blockIdx.y * tile_e) + 16 * l;
    unsigned char* ebuf = smem + 4 * X_TILE_BYTES;
    auto issue_exps = [&](int it, int buf) {   // past the last iteration the last one is re-read (nobody uses it)
        const int itc = it < nk ? it : nk - 1;
        if (w < 2) __builtin_amdgcn_global_load_lds((gptr)(xsrc + (int64_t)itc * 1024), (lptr)(ebuf + buf * X_EXP_BYTES + w * 1024), 16, 0, 0);
    };
    // this lane's four operand rows (x = 0, 1: tokens 64 wm + 32 x + c; x = 2, 3: channels 64 wn + 32 (x - 2) + c).  K
    // step kp (64 codes) uses block 2 kp + h; the MFMA picks a byte of a register by an immediate, the same for every
    // lane, so the half-wave h = 1 shifts its bytes down by one: byte 2 (kp & 1) of dword kp / 2 then is the block of
    // this lane.
    const int eoff[4] = {(64 * wm + c) * 8, (64 * wm + 32 + c) * 8, (XT + 64 * wn + c) * 8, (XT + 64 * wn + 32 + c) * 8};
    auto lds_exps = [&](int buf, u32x2 (&e)[4]) {
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const u32x2 v = *reinterpret_cast<const u32x2*>(ebuf + buf * X_EXP_BYTES + eoff[x]);
            e[x] = u32x2{v[0] >> (8 * h), v[1] >> (8 * h)};
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int aoff = (64 * wm + c) * XKB;
    const int boff = (64 * wn + c) * XKB;
    const int hs = h ^ ((c >> 1) & 7);   // chunk 2 kp + h of row 32 x + c sits in slot (2 kp) ^ hs
    constexpr int NKP = XKB / 32;        // K steps (64 codes) per tile
    static_assert(NKP == 4, "exponent bytes and the barrier position below");
    auto lds_chunk = [&](int buf, int kp, int x) -> u32x4 {
        const unsigned char* base = smem + ((x >> 1) * 2 + buf) * X_TILE_BYTES + ((x >> 1) ? boff : aoff);
        return *reinterpret_cast<const u32x4*>(base + 32 * (x & 1) * XKB + 16 * ((2 * kp) ^ hs));
    };
    auto mfma = [&](const u32x4& wv, const u32x4& xv, f32x16& cacc, int kp, const u32x2& ew, const u32x2& ex) {
        const i32x8 a = {(int)wv[0], (int)wv[1], (int)wv[2], (int)wv[3], 0, 0, 0, 0};
        const i32x8 b = {(int)xv[0], (int)xv[1], (int)xv[2], (int)xv[3], 0, 0, 0, 0};
        // formats: 4 = FP4 (E2M1) for both operands; byte 2 (kp & 1) of the exponent registers
        if (kp & 1) cacc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, cacc, 4, 4, 2, (int)ew[kp >> 1], 2, (int)ex[kp >> 1]);
        else cacc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, cacc, 4, 4, 0, (int)ew[kp >> 1], 0, (int)ex[kp >> 1]);
    };

    // Two-stage pipeline over K steps g = it * NKP + kp: while the MFMAs of step g run on P[g & 1], step g + 1 is read
    // from LDS into P[(g + 1) & 1].  Step NKP - 1 reads the first step of the next tile, so that tile is published
    // (loads waited for, barrier) after step NKP - 2; the buffer of the current tile is not read after that and
    // takes tile it + 2 behind the same barrier.
    u32x4 P[2][4];
    u32x2 E[2][4];   // exponents of the current and of the next tile
    issue(0, 0);
    issue_exps(0, 0);
    tile_ready();
    issue(1, 1);
    issue_exps(1, 1);
#pragma unroll
    for (int x = 0; x < 4; ++x) P[0][x] = lds_chunk(0, 0, x);
    lds_exps(0, E[0]);
    auto iteration = [&](int it, int buf, u32x2 (&ec)[4], u32x2 (&en)[4]) {
#pragma unroll
        for (int kp = 0; kp < NKP; ++kp) {
            const int cur = kp & 1, nxt = cur ^ 1;
            const int fkp = (kp + 1) % NKP;
            const int fbuf = (kp + 1 < NKP) ? buf : buf ^ 1;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int i = q >> 1, j = q & 1;
                mfma(P[cur][2 + j], P[cur][i], acc[i][j], kp, ec[2 + j], ec[i]);
                P[nxt][q] = lds_chunk(fbuf, fkp, q);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (kp == NKP - 2) {
                tile_ready();          // tile it + 1 and its exponents are in LDS; buffer `buf` is free
                lds_exps(buf ^ 1, en);
                issue(it + 2, buf);
                issue_exps(it + 2, buf);
            }
        }
    };
    for (int it = 0; it < nk; it += 2) {
        iteration(it, 0, E[0], E[1]);
        if (it + 1 < nk) iteration(it + 1, 1, E[1], E[0]);
    }
    tile_ready();   // no load is still writing, every wave is done with the K tiles: the epilogue reuses their space

    // epilogue: in acc[i][j] a lane holds, for token 64 wm + 32 i + c, the output channels 64 wn + 32 j + 8 (r / 4) + 4 h
    // + r % 4.  Rounded to fp16 and staged in LDS as a [128 tokens][128 channels] tile, which leaves in 16-byte pieces.
    typedef _Float16 half4 __attribute__((ext_vector_type(4)));
    constexpr int OPITCH = 2 * XT + 16;
    unsigned char* otile = smem;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int oc = 64 * wn + 32 * j + 8 * g + 4 * h;
                const half4 v = {(_Float16)acc[i][j][4 * g], (_Float16)acc[i][j][4 * g + 1], (_Float16)acc[i][j][4 * g + 2], (_Float16)acc[i][j][4 * g + 3]};
                *reinterpret_cast<half4*>(otile + (64 * wm + 32 * i + c) * OPITCH + 2 * oc) = v;
            }
    __syncthreads();
    const bool wide = ((reinterpret_cast<uintptr_t>(p.out) & 15) == 0) && (p.out_stride % 8 == 0);
#pragma unroll
    for (int k = 0; k < XT * 16 / X_NT; ++k) {
        const int q = tid + X_NT * k, row = q >> 4, ch = q & 15;
        const int64_t t = t0 + row;
        const int o = o0 + 8 * ch;
        if (t < p.T && o < p.m) {
            const u32x4 v = *reinterpret_cast<const u32x4*>(otile + row * OPITCH + 16 * ch);
            _Float16* dst = p.out + t * p.out_stride + o;
            if (wide && o + 8 <= p.m) {
                *reinterpret_cast<u32x4*>(dst) = v;
            } else {
                const _Float16* e = reinterpret_cast<const _Float16*>(&v);
                for (int x = 0; x < 8; ++x)
                    if (o + x < p.m) dst[x] = e[x];
            }
        }
    }
}

hipError_t mxfp4_gemm_launch(const MxGemmArgs& a, hipStream_t stream) {
    MxGemmDev d;
    d.xc = a.x_codes; d.xe = a.x_exps; d.wc = a.w_codes; d.we = a.w_exps; d.out = a.out;
    d.T = a.T; d.out_stride = a.out_stride; d.m = a.m; d.n = a.n;
    static OccCache cache;
    int unused = 0;
    hipError_t e = kernel_occupancy(reinterpret_cast<const void*>(mxfp4_gemm_kernel), X_NT, X_LDS_BYTES, cache, unused);
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)((a.T + XT - 1) / XT), (unsigned)((a.m + XT - 1) / XT));
    hipLaunchKernelGGL(mxfp4_gemm_kernel, grid, dim3(X_NT), X_LDS_BYTES, stream, d);
    return hipGetLastError();
}

}  // namespace fq
