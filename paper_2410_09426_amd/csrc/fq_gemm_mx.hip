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

// ---- few tokens (decode, short prefill chunks; tiles of up to 64 tokens): the weights are read once per tile and the kernel is bound by how fast a CU takes them in.  A
// workgroup owns 32 (or 16) output channels for all tokens; its waves split K by 128-byte lines (256 codes: wave w takes
// lines w, w + waves, ...) and each keeps a ring of line slots of its own in LDS: four global-to-LDS instructions
// bring 32 weight rows of a line (8 whole rows each), one per 8 token rows the tokens, one the 256 bytes of weight
// exponents (the tile order keeps them contiguous) and one per 32 tokens theirs.  A wave waits only for its own
// oldest slot (no barrier in the loop).  The partial sums of the waves are added in fp32 through LDS at the end.
// ROWS = 16: the workgroup owns 16 output channels only (twice as many workgroups, for layers with too few channels
// to give every CU one of 32); the MFMA's upper 16 rows repeat the lower ones and are dropped.
template <int NTD, int ROWS>   // token rows in groups of 8 (one load instruction each): 1, 2, 4, 8 for T <= 8, 16, 32, 64
__global__ __launch_bounds__(NTD >= 8 ? 512 : 1024) void mxfp4_skinny_kernel(MxGemmDev p, int depth) {
    static_assert(ROWS == 16 || ROWS == 32, "weight rows per workgroup");
    constexpr int NWI = ROWS / 8;                        // load instructions per line of the weight rows
    constexpr int NG = ROWS / 8;                         // groups of 8 output channels
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int NTT = NTD > 4 ? NTD / 4 : 1;           // MFMA token tiles of 32
    constexpr int XROWS = 8 * NTD;
    constexpr int XOFF = ROWS * 128, WEOFF = XOFF + 1024 * NTD, XEOFF = WEOFF + 256;
    constexpr int SLOT = XEOFF + 256 * NTT;
    constexpr int NI = NWI + NTD + 1 + NTT;              // load instructions per step
    const int tid = threadIdx.x;
    const int l = tid & 63, c = l & 31, h = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nwv = blockDim.x >> 6;
    const int o0 = blockIdx.x * ROWS;
    const int64_t t0 = (int64_t)blockIdx.y * XROWS;      // more than one token tile: launches past 64 tokens (tiles of 64)
    const int64_t kbytes = p.n / 2;
    const int nl = p.n / 256;                            // lines per row
    const int ns = (nl - w + nwv - 1) / nwv;             // this wave's steps
    unsigned char* ring = smem + w * depth * SLOT;

    const unsigned char* wsrc[NWI];
    const unsigned char* xsrc[NTD];
#pragma unroll
    for (int k = 0; k < NWI; ++k) {
        const int row = 8 * k + (l >> 3), ch = (l & 7) ^ ((row >> 1) & 7);
        int orow = o0 + row;
        if (orow >= p.m) orow = p.m - 1;
        wsrc[k] = p.wc + (int64_t)orow * kbytes + 128 * w + 16 * ch;
    }
#pragma unroll
    for (int k = 0; k < NTD; ++k) {
        const int row = 8 * k + (l >> 3), ch = (l & 7) ^ ((row >> 1) & 7);
        int64_t t = t0 + row;
        if (t >= p.T) t = p.T - 1;
        xsrc[k] = p.xc + t * kbytes + 128 * w + 16 * ch;
    }
    // exponents of line j: 1 KB per tile of 128 rows, 8 bytes per row.  The workgroup's 32 channels are 256 bytes of
    // their tile; the tokens are 32, 64 or 128 consecutive rows of one tile (the tensor is padded to whole tiles, so rows
    // past T exist).
    const unsigned char* wesrc = p.we + (int64_t)(o0 >> 7) * nl * 1024 + 8 * (o0 & 127) + 1024 * w + 4 * (l & (2 * ROWS - 1));
    const unsigned char* xesrc = p.xe + (t0 >> 7) * nl * 1024 + 8 * (t0 & 127) + 1024 * w + 4 * l;
    typedef const __attribute__((address_space(1))) void* gptr;
    typedef __attribute__((address_space(3))) void* lptr;
    auto issue = [&](int s, int slot) {
        unsigned char* base = ring + slot * SLOT;
        const int64_t off = (int64_t)s * (128 * nwv);
        const int64_t eoff = (int64_t)s * (1024 * nwv);
#pragma unroll
        for (int k = 0; k < NWI; ++k) __builtin_amdgcn_global_load_lds((gptr)(wsrc[k] + off), (lptr)(base + k * 1024), 16, 0, 0);
#pragma unroll
        for (int k = 0; k < NTD; ++k) __builtin_amdgcn_global_load_lds((gptr)(xsrc[k] + off), (lptr)(base + XOFF + k * 1024), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((gptr)(wesrc + eoff), (lptr)(base + WEOFF), 4, 0, 0);
#pragma unroll
        for (int i = 0; i < NTT; ++i) __builtin_amdgcn_global_load_lds((gptr)(xesrc + eoff + 256 * i), (lptr)(base + XEOFF + 256 * i), 4, 0, 0);
    };

    f32x16 acc[NTT];
#pragma unroll
    for (int i = 0; i < NTT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    const int woff = (c & (ROWS - 1)) * 128;
    const int whs = h ^ (((c & (ROWS - 1)) >> 1) & 7);
    int xoff[NTT], xhs[NTT];
#pragma unroll
    for (int i = 0; i < NTT; ++i) {
        const int row = (32 * i + c) & (XROWS - 1);       // fewer than 32 token rows: the lanes past them repeat rows
        xoff[i] = XOFF + row * 128;
        xhs[i] = h ^ ((row >> 1) & 7);
    }
    const int npre = ns < depth ? ns : depth;
    for (int s = 0; s < npre; ++s) issue(s, s);
    int slot = 0;
    for (int s = 0; s < ns; ++s) {
        const int left = ns - 1 - s;
        wait_ring_step<NI>(left < depth - 1 ? left : depth - 1);
        const unsigned char* base = ring + slot * SLOT;
        // block 2 kp + h of this lane's row: after the shift by 8 h, byte 2 (kp & 1) of dword kp / 2
        u32x2 ew = *reinterpret_cast<const u32x2*>(base + WEOFF + 8 * (c & (ROWS - 1)));
        ew = u32x2{ew[0] >> (8 * h), ew[1] >> (8 * h)};
        u32x2 ex[NTT];
#pragma unroll
        for (int i = 0; i < NTT; ++i) {
            const u32x2 v = *reinterpret_cast<const u32x2*>(base + XEOFF + 256 * i + 8 * c);
            ex[i] = u32x2{v[0] >> (8 * h), v[1] >> (8 * h)};
        }
        u32x4 wv[4], xv[4][NTT];
#pragma unroll
        for (int kp = 0; kp < 4; ++kp) {
            wv[kp] = *reinterpret_cast<const u32x4*>(base + woff + 16 * ((2 * kp) ^ whs));
#pragma unroll
            for (int i = 0; i < NTT; ++i) xv[kp][i] = *reinterpret_cast<const u32x4*>(base + xoff[i] + 16 * ((2 * kp) ^ xhs[i]));
        }
#pragma unroll
        for (int kp = 0; kp < 4; ++kp) {
            const i32x8 a = {(int)wv[kp][0], (int)wv[kp][1], (int)wv[kp][2], (int)wv[kp][3], 0, 0, 0, 0};
#pragma unroll
            for (int i = 0; i < NTT; ++i) {
                const i32x8 b = {(int)xv[kp][i][0], (int)xv[kp][i][1], (int)xv[kp][i][2], (int)xv[kp][i][3], 0, 0, 0, 0};
                if (kp & 1) acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[i], 4, 4, 2, (int)ew[kp >> 1], 2, (int)ex[i][kp >> 1]);
                else acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[i], 4, 4, 0, (int)ew[kp >> 1], 0, (int)ex[i][kp >> 1]);
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the slot has been read: it may take the next line
        if (s + depth < ns) issue(s + depth, slot);
        slot = (slot + 1 == depth) ? 0 : slot + 1;
    }
    wait_vm_pending<0>();
    __syncthreads();                                     // every wave is done with its ring: the partial sums go there
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    f32x4* part = reinterpret_cast<f32x4*>(smem);        // [wave][tile][quad g][lane] x 4 floats
#pragma unroll
    for (int i = 0; i < NTT; ++i)
#pragma unroll
        for (int g = 0; g < NG; ++g)
            part[((w * NTT + i) * NG + g) * 64 + l] = f32x4{acc[i][4 * g], acc[i][4 * g + 1], acc[i][4 * g + 2], acc[i][4 * g + 3]};
    __syncthreads();
    typedef _Float16 half4 __attribute__((ext_vector_type(4)));
    const bool wide = ((reinterpret_cast<uintptr_t>(p.out) & 7) == 0) && (p.out_stride % 4 == 0);
    for (int e = tid; e < NTT * NG * 64; e += (int)blockDim.x) {
        const int el = e & 63, g = (e >> 6) % NG, i = (e >> 6) / NG;
        f32x4 sum = part[e];
        for (int ww = 1; ww < nwv; ++ww) sum += part[ww * NTT * NG * 64 + e];
        const int64_t t = t0 + 32 * i + (el & 31);
        const int o = o0 + 8 * g + 4 * (el >> 5);
        if (t < p.T && o < p.m) {
            const _Float16 v[4] = {(_Float16)sum[0], (_Float16)sum[1], (_Float16)sum[2], (_Float16)sum[3]};
            _Float16* dst = p.out + t * p.out_stride + o;
            if (wide && o + 4 <= p.m) {
                *reinterpret_cast<half4*>(dst) = half4{v[0], v[1], v[2], v[3]};
            } else {
                for (int x = 0; x < 4; ++x)
                    if (o + x < p.m) dst[x] = v[x];
            }
        }
    }
}

template <int NTD, int ROWS>
static hipError_t mx_skinny_launch_rows(const MxGemmDev& d, hipStream_t stream, int token_tiles) {
    if (token_tiles < 1 || (token_tiles > 1 && NTD < 4)) return hipErrorInvalidValue;   // tiles of 32 tokens or more keep their exponents inside one 128-row tile
    static OccCache oc;
    int unused = 0;
    hipError_t e = kernel_occupancy(reinterpret_cast<const void*>(mxfp4_skinny_kernel<NTD, ROWS>), NTD >= 8 ? 512 : 1024, kRingLdsMax, oc, unused);
    if (e != hipSuccess) return e;
    constexpr int NTT = NTD > 4 ? NTD / 4 : 1;
    constexpr int SLOT = ROWS * 128 + 1024 * NTD + 256 + 256 * NTT, NI = ROWS / 8 + NTD + 1 + NTT;
    const unsigned wgx = (unsigned)((d.m + ROWS - 1) / ROWS);
    const int64_t wgs = (int64_t)wgx * token_tiles;
    const int nl = d.n / 256;
    // as for the INT4 product: 8 waves and two slots when there is at most one workgroup per CU, else 4 waves and one
    const bool crowded = wgs > cu_count();
    int nwv = env_int("FLATQUANT_GEMM_WAVES", crowded ? 4 : 8);
    int depth = env_int("FLATQUANT_GEMM_DEPTH", crowded ? 1 : 2);
    if ((nwv != 4 && nwv != 8 && nwv != 16) || depth < 1 || depth > kRingMaxDepth) return hipErrorInvalidValue;
    if (NTD >= 8 && nwv > 8) nwv = 8;                     // two token tiles of accumulators: compiled for at most 8 waves
    while (nwv > 4 && nwv * SLOT > kRingLdsMax) nwv >>= 1;
    const int steps = (nl + nwv - 1) / nwv;
    if (depth > steps) depth = steps;
    while (depth > 1 && (nwv * depth * SLOT > kRingLdsMax || (depth - 1) * NI > 63)) --depth;
    const int bytes = nwv * depth * SLOT;                // the partial sums (at most 4 KB per wave and token tile) reuse the rings
    return launch((mxfp4_skinny_kernel<NTD, ROWS>), dim3(wgx, (unsigned)token_tiles), dim3(64 * nwv), bytes, stream, d, depth);
}
// 16 channels per workgroup while that still leaves at most one workgroup per CU (FLATQUANT_GEMM_ROWS forces 16 or 32)
template <int NTD>
static hipError_t mx_skinny_launch(const MxGemmDev& d, hipStream_t stream, int token_tiles = 1) {
    const int rows = env_int("FLATQUANT_GEMM_ROWS", (int64_t)((d.m + 15) / 16) * token_tiles <= cu_count() ? 16 : 32);
    if (rows == 16) return mx_skinny_launch_rows<NTD, 16>(d, stream, token_tiles);
    if (rows == 32) return mx_skinny_launch_rows<NTD, 32>(d, stream, token_tiles);
    return hipErrorInvalidValue;
}

hipError_t mxfp4_gemm_launch(const MxGemmArgs& a, hipStream_t stream) {
    MxGemmDev d;
    d.xc = a.x_codes; d.xe = a.x_exps; d.wc = a.w_codes; d.we = a.w_exps; d.out = a.out;
    d.T = a.T; d.out_stride = a.out_stride; d.m = a.m; d.n = a.n;
    if (env_int("FLATQUANT_GEMM_TILED", 0) == 0) {
        // decode and short prefill chunks: one pass over the weights, K split inside a workgroup (the ring kernel)
        if (a.T <= 8) return mx_skinny_launch<1>(d, stream);
        if (a.T <= 16) return mx_skinny_launch<2>(d, stream);
        if (a.T <= 32) return mx_skinny_launch<4>(d, stream);
        if (a.T <= 64) return mx_skinny_launch<8>(d, stream);
        // More tokens: the ring kernel on tiles of 64 tokens, as long as the 128 x 128 tiles of the kernel below would
        // reach at most half of the CUs (measured cross-over on 1024 .. 11008 channels; FLATQUANT_GEMM_RING_MAX_T
        // replaces the rule by a token count).
        const int64_t tiled_wgs = ((a.T + XT - 1) / XT) * ((a.m + XT - 1) / XT);
        const int ring_max = env_int("FLATQUANT_GEMM_RING_MAX_T", -1);
        if (ring_max >= 0 ? a.T <= ring_max : (2 * tiled_wgs <= cu_count() && a.T <= 4096))
            return mx_skinny_launch<8>(d, stream, (int)((a.T + 63) / 64));
    }
    static OccCache cache;
    int unused = 0;
    hipError_t e = kernel_occupancy(reinterpret_cast<const void*>(mxfp4_gemm_kernel), X_NT, X_LDS_BYTES, cache, unused);
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)((a.T + XT - 1) / XT), (unsigned)((a.m + XT - 1) / XT));
    return launch(mxfp4_gemm_kernel, grid, dim3(X_NT), X_LDS_BYTES, stream, d);
}

}  // namespace fq
