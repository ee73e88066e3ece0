// W4A4 matrix product for gfx950: out[t, o] = fp16( s_x[t] s_w[o] sum_k q_x[t, k] q_w[o, k] ), the low-bit matrix
// multiplication that consumes the two quantized factors of Eq. (2) (Sec. 3.2: low-bit matrix multiplications for all
// linear layers; Sec. 3.3: the transform + quantization kernel feeds an INT4 GEMM).
//
// Both operands arrive as packed 4-bit two's-complement codes, K contiguous (activations [T, n/2], weights [m, n/2]),
// which is the operand order of an MFMA for C = A B^T.  The codes are widened to int8 on the fly without a sign
// extension: for a packed dword w, (w << 4) & 0xF0F0F0F0 holds 16 q of the even channels and w & 0xF0F0F0F0 holds 16 q
// of the odd channels, as signed bytes.  Both operands are widened the same way, so the K order inside an MFMA is
// the same permutation for both and every product carries a factor 256 that the epilogue divides out exactly.
// v_mfma_i32_32x32x32_i8 accumulates in int32 (|sum| <= 128 * 128 * n < 2^31 for n <= 65536).
//
// Workgroup: 4 waves, C tile 128 tokens x 128 output channels (or 8 waves, 256 x 128, when the launch has enough such
// tiles for every CU), each wave 64 x 64 (2 x 2 MFMA tiles; the weights are
// the MFMA's first operand so that a lane ends up with runs of 4 consecutive output channels of one token).  K advances by
// 256 codes (128 bytes = one cache line per row) per iteration through double-buffered LDS tiles, one barrier per
// iteration; the tiles go from global memory straight into LDS, a whole iteration before they are read.
// Launches whose 128 x 128 tiles would reach at most half of the CUs (decode, short prefill chunks) take the few-token
// kernel further down instead.
#include "fq_internal.h"

namespace fq {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int GT = 128;               // tile edge, tokens and output channels
constexpr int GKB = 128;              // packed bytes of K per row and iteration (256 codes)
constexpr int GPITCH = GKB;           // LDS row pitch: rows are written by global-to-LDS loads, 8 whole rows per wave and
                                      // instruction, so there is no padding; the 16-byte chunks of a row are swizzled instead
constexpr int G_NT = 256;
constexpr int G_TILE_BYTES = GT * GPITCH;
constexpr int G_LDS_BYTES = 4 * G_TILE_BYTES + GT * 4;   // A and B, two buffers each, + the weight steps of the tile
constexpr int G_LDS_BYTES_WIDE = 6 * G_TILE_BYTES + GT * 4;   // 256-token tile: A twice the size

struct GemmDev {
    const uint8_t* xc;
    const _Float16* xs;
    const uint8_t* wc;
    const _Float16* ws;
    _Float16* out;
    int64_t T;
    int64_t out_stride;
    int m, n;
};

// two k-steps of MFMA operands from 16 packed bytes
__device__ __forceinline__ void widen(const u32x4 w, i32x4& s0, i32x4& s1) {
    constexpr unsigned M = 0xF0F0F0F0u;
    s0 = i32x4{(int)((w[0] << 4) & M), (int)(w[0] & M), (int)((w[1] << 4) & M), (int)(w[1] & M)};
    s1 = i32x4{(int)((w[2] << 4) & M), (int)(w[2] & M), (int)((w[3] << 4) & M), (int)(w[3] & M)};
}

// TW = waves along the token axis: 2 -> C tile 128 tokens x 128 channels (4 waves), 4 -> 256 x 128 (8 waves): a quarter
// less operand traffic from L2 per product term, for launches with enough 256-token tiles to fill the chip.
template <int TW>
__global__ __launch_bounds__(128 * TW) __attribute__((amdgpu_waves_per_eu(2))) void w4a4_kernel(GemmDev p) {
    constexpr int GTM = 64 * TW;                       // tokens per tile
    constexpr int NW = 2 * TW;                         // waves
    constexpr int A_TILE = GTM * GPITCH, B_TILE = GT * GPITCH, STAGE = A_TILE + B_TILE;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x;
    const int l = tid & 63, c = l & 31, h = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w % TW, wn = w / TW;
    const int64_t t0 = (int64_t)blockIdx.x * GTM;
    const int o0 = blockIdx.y * GT;
    const int64_t kbytes = p.n / 2;
    const int nk = p.n / (2 * GKB);

    // Tile loads go from global memory straight into LDS (global_load_lds_dwordx4: lane i of a wave writes 16 bytes at
    // the wave's LDS base + 16 i, from any global address).  One instruction fills 8 rows of 128 bytes; wave w owns rows
    // 32 w .. 32 w + 31 of both tiles (4 instructions per operand and iteration).  LDS slot j of row r holds the row's
    // chunk j ^ ((r >> 1) & 7): with that swizzle the 16-byte operand reads of 32 consecutive rows (same chunk) spread
    // over all banks although the pitch is a multiple of the bank width.  Rows past the end re-read the last row.
    static_assert(GKB == 128 && GT == 128, "load mapping below");
    constexpr int NLA = GTM / 8 / NW, NLB = GT / 8 / NW;   // 8-row instructions per wave: 4 and 4 (4 waves), 4 and 2 (8 waves)
    const unsigned char* asrc[NLA];
    const unsigned char* bsrc[NLB];
#pragma unroll
    for (int k = 0; k < NLA; ++k) {
        const int row = 8 * (NLA * w + k) + (l >> 3), ch = (l & 7) ^ ((row >> 1) & 7);
        int64_t tr = t0 + row;
        if (tr >= p.T) tr = p.T - 1;
        asrc[k] = p.xc + tr * kbytes + 16 * ch;
    }
#pragma unroll
    for (int k = 0; k < NLB; ++k) {
        const int row = 8 * (NLB * w + k) + (l >> 3), ch = (l & 7) ^ ((row >> 1) & 7);
        int orow = o0 + row;
        if (orow >= p.m) orow = p.m - 1;
        bsrc[k] = p.wc + (int64_t)orow * kbytes + 16 * ch;
    }
    typedef const __attribute__((address_space(1))) void* gptr;
    typedef __attribute__((address_space(3))) void* lptr;
    auto issue = [&](int it, int buf) {   // past the last tile the last one is re-read (nobody uses it): no branch in the loop body
        const int itc = it < nk ? it : nk - 1;
        unsigned char* A = smem + buf * STAGE + w * (8 * NLA * GPITCH);
        unsigned char* B = smem + buf * STAGE + A_TILE + w * (8 * NLB * GPITCH);
#pragma unroll
        for (int k = 0; k < NLA; ++k) __builtin_amdgcn_global_load_lds((gptr)(asrc[k] + (int64_t)itc * GKB), (lptr)(A + k * 8 * GPITCH), 16, 0, 0);
#pragma unroll
        for (int k = 0; k < NLB; ++k) __builtin_amdgcn_global_load_lds((gptr)(bsrc[k] + (int64_t)itc * GKB), (lptr)(B + k * 8 * GPITCH), 16, 0, 0);
    };
    // the tile requested last has arrived in LDS (this wave's part), then every wave's part has
    auto tile_ready = [&]() {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    };

    i32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    if (tid < GT) {
        const int o = o0 + tid;
        reinterpret_cast<float*>(smem + 2 * STAGE)[tid] = (o < p.m) ? (float)p.ws[o] : 0.0f;
    }
    const int aoff = (64 * wm + c) * GPITCH;
    const int boff = (64 * wn + c) * GPITCH;
    const int hs = h ^ ((c >> 1) & 7);   // chunk 2 kp + h of row 32 x + c sits in slot (2 kp) ^ hs (the row's swizzle is that of c)
    constexpr int NKP = GKB / 32;   // K step pairs (64 codes) per tile
    static_assert(NKP >= 4 && NKP % 2 == 0, "the pipeline below reads two step pairs ahead and alternates two register stages");
    // packed operands of one K step pair: x = 0, 1: tokens 32 x + c (A); x = 2, 3: output channels 32 (x - 2) + c (B)
    auto lds_chunk = [&](int buf, int kp, int x) -> u32x4 {
        const unsigned char* base = smem + buf * STAGE + ((x >> 1) ? A_TILE + boff : aoff);
        return *reinterpret_cast<const u32x4*>(base + 32 * (x & 1) * GPITCH + 16 * ((2 * kp) ^ hs));
    };
    // Software pipeline over K step pairs g = it * NKP + kp, three stages deep: while the MFMAs of pair g run on the
    // widened operands W[g & 1], pair g + 1 is widened from its packed registers P[(g + 1) & 1] into W[(g + 1) & 1] and
    // pair g + 2 is read from LDS into P[g & 1].  The work is cut into 8 slices per pair, one MFMA followed by one
    // slice of widening (6 vector instructions, shorter than the MFMA) and at most one LDS read, in this order in
    // the instruction stream: a wave issues in order, so only vector work that sits between two MFMAs can run in
    // the shadow of the first.
    u32x4 P[2][4];
    i32x4 W[2][4][2];   // [stage][operand x][K step s]
    issue(0, 0);
    tile_ready();
    issue(1, 1);
#pragma unroll
    for (int x = 0; x < 4; ++x) { P[0][x] = lds_chunk(0, 0, x); P[1][x] = lds_chunk(0, 1, x); }
    constexpr unsigned M = 0xF0F0F0F0u;
    auto widen_slice = [&](const u32x4& w, int s) -> i32x4 {
        return i32x4{(int)((w[2 * s] << 4) & M), (int)(w[2 * s] & M), (int)((w[2 * s + 1] << 4) & M), (int)(w[2 * s + 1] & M)};
    };
#pragma unroll
    for (int x = 0; x < 4; ++x) { W[0][x][0] = widen_slice(P[0][x], 0); W[0][x][1] = widen_slice(P[0][x], 1); }
    // one iteration: tile `it` (LDS buffer `buf`) through the MFMAs.  After pair NKP - 3 nobody reads that buffer any
    // more (the later pairs were read ahead), so behind the barrier that publishes tile it + 1 it takes tile it + 2.
    auto iteration = [&](int it, int buf) {
#pragma unroll
        for (int kp = 0; kp < NKP; ++kp) {
            const int cur = kp & 1, nxt = cur ^ 1;           // NKP is even: the stage parity of pair g is that of kp
            const int fkp = (kp + 2) % NKP;                   // pair g + 2: in this tile, or the first pairs of the next one
            const int fbuf = (kp + 2 < NKP) ? buf : buf ^ 1;
#pragma unroll
            for (int m = 0; m < 8; ++m) {
                const int s = m >> 2, i = (m >> 1) & 1, j = m & 1;
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(W[cur][2 + j][s], W[cur][i][s], acc[i][j], 0, 0, 0);
                W[nxt][m >> 1][m & 1] = widen_slice(P[nxt][m >> 1], m & 1);
                // P[cur] was widened during the previous pair: its registers take pair g + 2
                if (m >= 4) P[cur][m - 4] = lds_chunk(fbuf, fkp, m - 4);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (kp == NKP - 3) {
                tile_ready();
                issue(it + 2, buf);
            }
        }
    };
    for (int it = 0; it < nk; it += 2) {
        iteration(it, 0);
        if (it + 1 < nk) iteration(it + 1, 1);
    }
    tile_ready();   // no load is still writing, every wave is done with the K tiles: the epilogue reuses their space

    // epilogue.  The weights are the MFMA's first operand, so in acc[i][j] a lane holds, for token 64 wm + 32 i + c,
    // the output channels 64 wn + 32 j + 8 (r / 4) + 4 h + r % 4: runs of 4 consecutive channels.  They are scaled,
    // rounded to fp16 and staged in LDS (the K tiles are dead by now) as a [128 tokens][128 channels] tile, which then
    // leaves in whole 16-byte pieces.  Every sum is a multiple of 256 (both operands carry a factor 16).
    typedef _Float16 half4 __attribute__((ext_vector_type(4)));
    constexpr int OPITCH = 2 * GT + 16;
    unsigned char* otile = smem;
    float* sws = reinterpret_cast<float*>(smem + 2 * STAGE);          // [128] weight steps of this tile
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int64_t t = t0 + 64 * wm + 32 * i + c;
        const float sx = (float)p.xs[t < p.T ? t : p.T - 1];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int oc = 64 * wn + 32 * j + 8 * g + 4 * h;
                const float4 sw = *reinterpret_cast<const float4*>(sws + oc);
                const half4 v = {(_Float16)((float)(acc[i][j][4 * g] >> 8) * sx * sw.x), (_Float16)((float)(acc[i][j][4 * g + 1] >> 8) * sx * sw.y),
                                 (_Float16)((float)(acc[i][j][4 * g + 2] >> 8) * sx * sw.z), (_Float16)((float)(acc[i][j][4 * g + 3] >> 8) * sx * sw.w)};
                *reinterpret_cast<half4*>(otile + (64 * wm + 32 * i + c) * OPITCH + 2 * oc) = v;
            }
    }
    __syncthreads();
    const bool wide = ((reinterpret_cast<uintptr_t>(p.out) & 15) == 0) && (p.out_stride % 8 == 0);
#pragma unroll
    for (int k = 0; k < GTM * 16 / (64 * NW); ++k) {
        const int q = tid + 64 * NW * k, row = q >> 4, ch = q & 15;
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

// ---- few tokens (decode, short prefill chunks): the weights are read once (per tile of 64 tokens), and what bounds the kernel is how fast the CUs take
// them in.  A workgroup owns 32 (or 16) output channels for all tokens.  Every operand byte goes from global memory
// straight into LDS, a whole cache line per row at a time: a wave owns every nwv-th 128-byte line of K (256 codes) of
// the workgroup's weight rows and of the token rows, with a ring of `depth` line slots of its own in LDS.  One
// global-to-LDS instruction moves 8 whole rows; the wave waits only for its own oldest slot (no barrier in the loop),
// multiplies it and requests the line `depth` steps ahead into the same slot.  The slots use the swizzle of the tiled
// kernel (slot chunk j of row r holds the row's chunk j ^ ((r >> 1) & 7)).  The partial sums of the waves are added
// through LDS at the end.  (Feeding the MFMA from registers instead, 32 bytes of 32 rows per load, costs four
// instructions and tag look-ups per cache line and holds far less in flight: 1.5 to 3 times slower.)
// ROWS = 16: the workgroup owns 16 output channels only (twice as many workgroups, for layers with too few channels
// to give every CU one of 32); the MFMA's upper 16 rows repeat the lower ones and are dropped.
template <int NTD, int ROWS>   // token rows in groups of 8 (one load instruction each): 1, 2, 4, 8 for T <= 8, 16, 32, 64
__global__ __launch_bounds__(NTD >= 8 ? 512 : 1024) void w4a4_skinny_kernel(GemmDev p, int depth) {
    static_assert(ROWS == 16 || ROWS == 32, "weight rows per workgroup");
    constexpr int NWI = ROWS / 8;                        // load instructions per line of the weight rows
    constexpr int NG = ROWS / 8;                         // groups of 8 output channels
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int NTT = NTD > 4 ? NTD / 4 : 1;           // MFMA token tiles of 32
    constexpr int XROWS = 8 * NTD;
    constexpr int XOFF = ROWS * 128;
    constexpr int SLOT = (ROWS + XROWS) * 128;           // weight rows, then token rows, one line each
    constexpr int NI = NWI + NTD;                        // load instructions per step
    const int tid = threadIdx.x;
    const int l = tid & 63, c = l & 31, h = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int o0 = blockIdx.x * ROWS;
    const int64_t t0 = (int64_t)blockIdx.y * XROWS;      // more than one token tile: launches past 64 tokens (tiles of 64)
    const int64_t kbytes = p.n / 2;
    const int nl = p.n / 256;                            // lines per row
    const int nwv = blockDim.x >> 6;                     // waves: 4, 8 or 16
    const int ns = (nl - w + nwv - 1) / nwv;             // this wave's steps: lines w, w + nwv, ...
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
    typedef const __attribute__((address_space(1))) void* gptr;
    typedef __attribute__((address_space(3))) void* lptr;
    auto issue = [&](int s, int slot) {
        unsigned char* base = ring + slot * SLOT;
        const int64_t off = (int64_t)s * (128 * nwv);
#pragma unroll
        for (int k = 0; k < NWI; ++k) __builtin_amdgcn_global_load_lds((gptr)(wsrc[k] + off), (lptr)(base + k * 1024), 16, 0, 0);
#pragma unroll
        for (int k = 0; k < NTD; ++k) __builtin_amdgcn_global_load_lds((gptr)(xsrc[k] + off), (lptr)(base + XOFF + k * 1024), 16, 0, 0);
    };
    i32x16 acc[NTT];
#pragma unroll
    for (int i = 0; i < NTT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;
    const int woff = (c & (ROWS - 1)) * 128;
    const int whs = h ^ (((c & (ROWS - 1)) >> 1) & 7);
    int xoff[NTT], xhs[NTT];
#pragma unroll
    for (int i = 0; i < NTT; ++i) {
        const int row = (32 * i + c) & (XROWS - 1);       // fewer than 32 token rows: the lanes past them repeat rows
        xoff[i] = XOFF + row * 128;
        xhs[i] = h ^ ((row >> 1) & 7);
    }
    // The epilogue's element e = tid + k blockDim is 4 output channels of one token: their steps are requested now, so
    // that the kernel's tail does not wait for them (at least 256 threads: k < NK).
    constexpr int NE = NTT * NG * 64;
    constexpr int NK = (NE + 255) / 256;
    unsigned esx[NK] = {}, esw[NK][4] = {};              // raw fp16 bits, converted in the epilogue: nothing waits for them here
    const uint16_t* xs_bits = reinterpret_cast<const uint16_t*>(p.xs);
    const uint16_t* ws_bits = reinterpret_cast<const uint16_t*>(p.ws);
#pragma unroll
    for (int k = 0; k < NK; ++k) {
        const int e = tid + k * (int)blockDim.x;
        const int el = e & 63, g = (e >> 6) % NG, i = (e >> 6) / NG;
        const int64_t t = t0 + 32 * i + (el & 31);
        const int o = o0 + 8 * g + 4 * (el >> 5);
        if (e < NE) {
            esx[k] = xs_bits[t < p.T ? t : p.T - 1];
#pragma unroll
            for (int x = 0; x < 4; ++x) esw[k][x] = ws_bits[o + x < p.m ? o + x : p.m - 1];
        }
    }
    const int npre = ns < depth ? ns : depth;
    for (int s = 0; s < npre; ++s) issue(s, s);
    int slot = 0;
    for (int s = 0; s < ns; ++s) {
        const int left = ns - 1 - s;
        wait_ring_step<NI>(left < depth - 1 ? left : depth - 1);
        const unsigned char* base = ring + slot * SLOT;
        u32x4 wv[4], xv[4][NTT];
#pragma unroll
        for (int kp = 0; kp < 4; ++kp) {
            wv[kp] = *reinterpret_cast<const u32x4*>(base + woff + 16 * ((2 * kp) ^ whs));
#pragma unroll
            for (int i = 0; i < NTT; ++i) xv[kp][i] = *reinterpret_cast<const u32x4*>(base + xoff[i] + 16 * ((2 * kp) ^ xhs[i]));
        }
#pragma unroll
        for (int kp = 0; kp < 4; ++kp) {
            i32x4 ws0, ws1;
            widen(wv[kp], ws0, ws1);
#pragma unroll
            for (int i = 0; i < NTT; ++i) {
                i32x4 xs0, xs1;
                widen(xv[kp][i], xs0, xs1);
                acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ws0, xs0, acc[i], 0, 0, 0);
                acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ws1, xs1, acc[i], 0, 0, 0);
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the slot has been read: it may take the next line
        if (s + depth < ns) issue(s + depth, slot);
        slot = (slot + 1 == depth) ? 0 : slot + 1;
    }
    wait_vm_pending<0>();
    __syncthreads();                                     // every wave is done with its ring: the partial sums go there
    i32x4* part = reinterpret_cast<i32x4*>(smem);
#pragma unroll
    for (int i = 0; i < NTT; ++i)
#pragma unroll
        for (int g = 0; g < NG; ++g)
            part[((w * NTT + i) * NG + g) * 64 + l] = i32x4{acc[i][4 * g], acc[i][4 * g + 1], acc[i][4 * g + 2], acc[i][4 * g + 3]};
    __syncthreads();
    typedef _Float16 half4 __attribute__((ext_vector_type(4)));
    const bool wide = ((reinterpret_cast<uintptr_t>(p.out) & 7) == 0) && (p.out_stride % 4 == 0);
#pragma unroll
    for (int k = 0; k < NK; ++k) {
        const int e = tid + k * (int)blockDim.x;
        if (e >= NE) break;
        const int el = e & 63, g = (e >> 6) % NG, i = (e >> 6) / NG;
        i32x4 sum = part[e];
        for (int ww = 1; ww < nwv; ++ww) sum += part[ww * NE + e];
        const int64_t t = t0 + 32 * i + (el & 31);
        const int o = o0 + 8 * g + 4 * (el >> 5);
        if (t < p.T && o < p.m) {
            // (the empty statement pins the conversions here: hoisted to the loads, they would stall the kernel's start)
            asm volatile("" : "+v"(esx[k]), "+v"(esw[k][0]), "+v"(esw[k][1]), "+v"(esw[k][2]), "+v"(esw[k][3]));
            const float sx = (float)__builtin_bit_cast(_Float16, (uint16_t)esx[k]);
            _Float16 v[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) v[x] = (_Float16)((float)(sum[x] >> 8) * sx * (float)__builtin_bit_cast(_Float16, (uint16_t)esw[k][x]));
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
static hipError_t skinny_launch_rows(const GemmDev& d, hipStream_t stream, int token_tiles) {
    if (token_tiles < 1 || (token_tiles > 1 && NTD < 4)) return hipErrorInvalidValue;   // tiles of 32 tokens or more keep their exponents inside one 128-row tile
    static OccCache oc;
    int unused = 0;
    hipError_t e = kernel_occupancy(reinterpret_cast<const void*>(w4a4_skinny_kernel<NTD, ROWS>), NTD >= 8 ? 512 : 1024, kRingLdsMax, oc, unused);
    if (e != hipSuccess) return e;
    constexpr int SLOT = (ROWS + 8 * NTD) * 128, NI = ROWS / 8 + NTD;
    const unsigned wgx = (unsigned)((d.m + ROWS - 1) / ROWS);
    const int64_t wgs = (int64_t)wgx * token_tiles;
    const int nl = d.n / 256;
    // One workgroup per CU (or fewer): 8 waves, so that every SIMD has two to overlap, and two slots each.  More than
    // one per CU: small workgroups (4 waves, one slot) that are all resident at once; what the second slot or the
    // other four waves would hide, the neighbouring workgroup hides.  (Measured on 4096 / 11008-wide layers.)
    const bool crowded = wgs > cu_count();
    int nwv = env_int("FLATQUANT_GEMM_WAVES", crowded ? 4 : 8);
    int depth = env_int("FLATQUANT_GEMM_DEPTH", crowded ? 1 : 2);
    if ((nwv != 4 && nwv != 8 && nwv != 16) || depth < 1 || depth > kRingMaxDepth) return hipErrorInvalidValue;
    if (NTD >= 8 && nwv > 8) nwv = 8;                                      // two token tiles of accumulators: compiled for at most 8 waves
    while (nwv > 4 && nwv * SLOT > kRingLdsMax) nwv >>= 1;
    const int steps = (nl + nwv - 1) / nwv;                               // of the wave with the most lines
    if (depth > steps) depth = steps;
    while (depth > 1 && (nwv * depth * SLOT > kRingLdsMax || (depth - 1) * NI > 63)) --depth;
    const int bytes = nwv * depth * SLOT;                                 // the partial sums (at most 4 KB per wave and token tile) reuse the rings
    return launch((w4a4_skinny_kernel<NTD, ROWS>), dim3(wgx, (unsigned)token_tiles), dim3(64 * nwv), bytes, stream, d, depth);
}
// 16 channels per workgroup while that still leaves at most one workgroup per CU (FLATQUANT_GEMM_ROWS forces 16 or 32):
// the kernel is bound by what one CU takes in, so the channels go to as many CUs as there are.
template <int NTD>
static hipError_t skinny_launch(const GemmDev& d, hipStream_t stream, int token_tiles = 1) {
    const int rows = env_int("FLATQUANT_GEMM_ROWS", (int64_t)((d.m + 15) / 16) * token_tiles <= cu_count() ? 16 : 32);
    if (rows == 16) return skinny_launch_rows<NTD, 16>(d, stream, token_tiles);
    if (rows == 32) return skinny_launch_rows<NTD, 32>(d, stream, token_tiles);
    return hipErrorInvalidValue;
}

hipError_t w4a4_launch(const GemmArgs& a, hipStream_t stream) {
    int unused = 0;
    GemmDev d;
    d.xc = a.x_codes; d.xs = a.x_scales; d.wc = a.w_codes; d.ws = a.w_scales; d.out = a.out;
    d.T = a.T; d.out_stride = a.out_stride; d.m = a.m; d.n = a.n;
    if (env_int("FLATQUANT_GEMM_TILED", 0) == 0) {
        // decode and short prefill chunks: one pass over the weights, K split inside a workgroup (the ring kernel)
        if (a.T <= 8) return skinny_launch<1>(d, stream);
        if (a.T <= 16) return skinny_launch<2>(d, stream);
        if (a.T <= 32) return skinny_launch<4>(d, stream);
        if (a.T <= 64) return skinny_launch<8>(d, stream);
        // More tokens: the ring kernel on tiles of 64 tokens, as long as the 128 x 128 tiles of the kernel below would
        // reach at most half of the CUs (measured cross-over on 1024 .. 11008 channels; FLATQUANT_GEMM_RING_MAX_T
        // replaces the rule by a token count).
        const int64_t tiled_wgs = ((a.T + GT - 1) / GT) * ((a.m + GT - 1) / GT);
        const int ring_max = env_int("FLATQUANT_GEMM_RING_MAX_T", -1);
        if (ring_max >= 0 ? a.T <= ring_max : (2 * tiled_wgs <= cu_count() && a.T <= 4096))
            return skinny_launch<8>(d, stream, (int)((a.T + 63) / 64));
    }
    static OccCache ct, ctw;
    // 256-token tiles when they still give every CU a workgroup (FLATQUANT_GEMM_WIDE = 0 / 1 forces a form)
    const int64_t wide_wgs = ((a.T + 255) / 256) * ((a.m + GT - 1) / GT);
    const int wide = env_int("FLATQUANT_GEMM_WIDE", wide_wgs >= cu_count() ? 1 : 0);
    if (wide) {
        hipError_t e = kernel_occupancy(reinterpret_cast<const void*>(w4a4_kernel<4>), 512, G_LDS_BYTES_WIDE, ctw, unused);
        if (e != hipSuccess) return e;
        const dim3 grid((unsigned)((a.T + 255) / 256), (unsigned)((a.m + GT - 1) / GT));
        return launch(w4a4_kernel<4>, grid, dim3(512), G_LDS_BYTES_WIDE, stream, d);
    }
    {
        hipError_t e = kernel_occupancy(reinterpret_cast<const void*>(w4a4_kernel<2>), G_NT, G_LDS_BYTES, ct, unused);
        if (e != hipSuccess) return e;
    }
    const dim3 grid((unsigned)((a.T + GT - 1) / GT), (unsigned)((a.m + GT - 1) / GT));
    return launch(w4a4_kernel<2>, grid, dim3(G_NT), G_LDS_BYTES, stream, d);
}

}  // namespace fq
