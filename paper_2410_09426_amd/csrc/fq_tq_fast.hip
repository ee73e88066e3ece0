// Specialised fused transform + INT4 kernels for gfx950: n2 a multiple of 32 and
// 16-byte aligned rows, so that every shape test is resolved at compile time.
//
// Same method and same wave mapping as the general kernel in
// fq_transform_quant.hip (Eq. (2) left factor, fused as in Sec. 3.3): one wave
// per 32-column slab of n2; Z = X~ P2[:, slab] on MFMA with the token tile as A
// operand from LDS; Y^T = Z^T P1 on MFMA with Z's accumulators, split into fp16
// hi + lo, fed back as the A operand; per-token absmax; clip; round; pack; store.
// What is different here:
//   * P1 and P2 are fetched with coalesced 16-byte loads into LDS once per
//     workgroup and the strided MFMA fragments are gathered from LDS, not HBM/L2.
//   * The loop body has no shape conditionals, the wave reduction uses DPP, and
//     rounding + nibble extraction is one fused multiply-add against 1.5 * 2^23.
#include "fq_internal.h"

namespace fq {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__host__ __device__ constexpr int cmax(int a, int b) { return a > b ? a : b; }

// LDS carve-up, shared by host and device.
template <int A, int B>
struct FastLds {
    static constexpr int N2 = 32 * B;
    static constexpr int PITCH = N2 + kLdsPad;                       // halves per row of the token tile
    static constexpr int XS_BYTES = 32 * A * PITCH * 2;
    static constexpr int STAGE_BYTES = 512 * A * B;                  // packed codes of one token
    static constexpr int BODY_BYTES = XS_BYTES + STAGE_BYTES + 32;   // + one absmax float per wave
    static constexpr int P2ROWS = (B <= 4) ? N2 : N2 / 2;            // rows of P2 staged per pass
    static constexpr int P2PASSES = N2 / P2ROWS;
    static constexpr int P1FLAT_BYTES = 32 * A * 32 * A * 2;
    static constexpr int STG_BYTES = P1FLAT_BYTES + P2ROWS * N2 * 2;
    static constexpr int R0 = (cmax(BODY_BYTES, STG_BYTES) + 15) & ~15;
    static constexpr bool P1LDS = (A >= 3);
    static constexpr int P1S_BYTES = P1LDS ? A * 2 * A * 64 * 16 : 0;
    static constexpr int TOTAL = R0 + P1S_BYTES;
};

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

// fp32 x8 -> fp16 hi (round toward zero, cannot overflow to inf) and fp16 lo = fp16(z - hi)
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

template <int A, int B, bool FULL1>
__global__ __launch_bounds__(64 * B) __attribute__((amdgpu_waves_per_eu(2))) void tq_fast_kernel(TqDev p) {
    using L = FastLds<A, B>;
    constexpr int NT = 64 * B, N2 = L::N2, PITCH = L::PITCH;
    constexpr int KB1 = 2 * A, KB2 = 2 * B, NPRE = 2 * A;
    constexpr int CPR = 4 * B;                    // 16-byte chunks per row of X~
    constexpr bool P1LDS = L::P1LDS;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    _Float16* Xs = reinterpret_cast<_Float16*>(smem);
    uint8_t* stage = smem + L::XS_BYTES;
    float* red = reinterpret_cast<float*>(stage + L::STAGE_BYTES);
    u32x4* P1s = reinterpret_cast<u32x4*>(smem + L::R0);
    _Float16* P1flat = reinterpret_cast<_Float16*>(smem);
    _Float16* P2flat = reinterpret_cast<_Float16*>(smem + L::P1FLAT_BYTES);

    const int tid = threadIdx.x;
    const int l = tid & 63, w = tid >> 6, c = l & 31, h = l >> 5;
    const int n1 = FULL1 ? 32 * A : p.n1;
    const int64_t row_bytes_out = (int64_t)n1 * (N2 / 2);

    // chunk k of this thread: row (tid / CPR) + 16k of X~, 8 halves at column (tid % CPR) * 8
    const int xrow0 = tid / CPR;
    const int xbase = xrow0 * PITCH + (tid % CPR) * 8;

    auto issue = [&](int64_t t, u32x4 (&pre)[NPRE]) {
        const u32x4* src = reinterpret_cast<const u32x4*>(p.x + t * p.x_stride) + tid;
#pragma unroll
        for (int k = 0; k < NPRE; ++k)
            if (FULL1 || xrow0 + 16 * k < n1) pre[k] = __builtin_nontemporal_load(src + k * NT);
    };
    auto commit = [&](const u32x4 (&pre)[NPRE]) {
#pragma unroll
        for (int k = 0; k < NPRE; ++k)
            if (FULL1 || xrow0 + 16 * k < n1) *reinterpret_cast<u32x4*>(Xs + xbase + 16 * k * PITCH) = pre[k];
    };

    // ---- the first two token rows of this workgroup are requested before anything else
    constexpr bool DEEP = (A <= 2);   // two rows in flight per workgroup when the registers allow it
    u32x4 pre0[NPRE], pre1[DEEP ? NPRE : 1];
    int64_t t = blockIdx.x;
    const int64_t G = gridDim.x;
    issue(t, pre0);
    if constexpr (DEEP) {
        if (t + G < p.T) issue(t + G, pre1);
    }

    // ---- stage P1 (flat, n1 x n1) and the first pass of P2 rows in LDS with coalesced loads
    {
        const int n1sq = n1 * n1;
        if ((n1sq & 7) == 0) {
            for (int q = tid; q < (n1sq >> 3); q += NT)
                reinterpret_cast<u32x4*>(P1flat)[q] = reinterpret_cast<const u32x4*>(p.P1)[q];
        } else {   // n1 * n1 not a multiple of 8 halves: pairs, plus a last odd element
            for (int q = tid; q < (n1sq >> 1); q += NT)
                reinterpret_cast<uint32_t*>(P1flat)[q] = reinterpret_cast<const uint32_t*>(p.P1)[q];
            if ((n1sq & 1) && tid == 0) P1flat[n1sq - 1] = p.P1[n1sq - 1];
        }
    }
    half8 p2f[KB2];
    half8 p1f[P1LDS ? 1 : A][P1LDS ? 1 : KB1];
#pragma unroll
    for (int pass = 0; pass < L::P2PASSES; ++pass) {
        if (pass > 0) __syncthreads();   // previous pass fully consumed
        constexpr int CH = L::P2ROWS * N2 / 8;
        const u32x4* src = reinterpret_cast<const u32x4*>(p.P2) + pass * CH;
#pragma unroll
        for (int k = 0; k < CH / NT; ++k) reinterpret_cast<u32x4*>(P2flat)[tid + k * NT] = src[tid + k * NT];
        __syncthreads();
        // B-operand fragments of this wave's slab: lane (c, h) holds P2[16kb + 8h + s][32w + c], s = 0..7
#pragma unroll
        for (int kb = pass * (L::P2ROWS / 16); kb < (pass + 1) * (L::P2ROWS / 16); ++kb)
#pragma unroll
            for (int s = 0; s < 8; ++s)
                p2f[kb][s] = P2flat[(16 * kb - pass * L::P2ROWS + 8 * h + s) * N2 + 32 * w + c];
        if (pass == 0) {
            // P1 fragments, gathered with the k-permutation of the first contraction's accumulator layout:
            // K block kk, slot s, half-wave h  <->  i = 32(kk/2) + 8(2(kk%2) + s/4) + 4h + s%4
            if constexpr (P1LDS) {
                for (int e = tid; e < A * KB1 * 64; e += NT) {
                    const int ln = e & 63, kk = (e >> 6) % KB1, It = (e >> 6) / KB1;
                    const int cc = ln & 31, hh = ln >> 5, ip = 32 * It + cc;
                    half8 f;
#pragma unroll
                    for (int s = 0; s < 8; ++s) {
                        const int i = 32 * (kk >> 1) + 8 * (2 * (kk & 1) + (s >> 2)) + 4 * hh + (s & 3);
                        f[s] = (FULL1 || (i < n1 && ip < n1)) ? P1flat[i * n1 + ip] : (_Float16)0;
                    }
                    *reinterpret_cast<half8*>(&P1s[e]) = f;
                }
            } else {
#pragma unroll
                for (int It = 0; It < A; ++It)
#pragma unroll
                    for (int kk = 0; kk < KB1; ++kk) {
                        const int ip = 32 * It + c;
#pragma unroll
                        for (int s = 0; s < 8; ++s) {
                            const int i = 32 * (kk >> 1) + 8 * (2 * (kk & 1) + (s >> 2)) + 4 * h + (s & 3);
                            p1f[It][kk][s] = (FULL1 || (i < n1 && ip < n1)) ? P1flat[i * n1 + ip] : (_Float16)0;
                        }
                    }
            }
        }
    }
    __syncthreads();   // staging area is free: it becomes the token tile
    if constexpr (!FULL1) {   // rows n1 .. 32A-1 of the tile are never loaded: make them exact zeros once
        for (int q = tid; q < (32 * A - n1) * (PITCH / 8); q += NT)
            reinterpret_cast<u32x4*>(Xs + n1 * PITCH)[q] = u32x4{0u, 0u, 0u, 0u};
    }
    commit(pre0);
    __syncthreads();

    // One token: the tile of token t is in LDS, `pre_next` holds (or is receiving) the row of token t + G and is
    // written to LDS once every wave is done with the current tile; the row of token t + 2G is requested into
    // `pre_far`.  The caller alternates the two register sets.
    auto body = [&](int64_t t, u32x4 (&pre_next)[NPRE], u32x4 (&pre_far)[NPRE]) {
        const bool have_next = t + G < p.T;
        if (t + (DEEP ? 2 : 1) * G < p.T) issue(t + (DEEP ? 2 : 1) * G, pre_far);
        const float clipv = p.clip[p.clip_mode ? t : 0];

        f32x16 acc2[A];
#pragma unroll
        for (int It = 0; It < A; ++It)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc2[It][r] = 0.0f;

        // row tiles of X~ go through the first contraction in pairs so that consecutive MFMAs are independent
#pragma unroll
        for (int I0 = 0; I0 < A; I0 += 2) {
            constexpr int NI_MAX = 2;
            const int ni = (A - I0) < NI_MAX ? (A - I0) : NI_MAX;
            f32x16 acc1[NI_MAX];
#pragma unroll
            for (int d = 0; d < NI_MAX; ++d)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc1[d][r] = 0.0f;
            const _Float16* arow = Xs + (32 * I0 + c) * PITCH + 8 * h;
#pragma unroll
            for (int kb = 0; kb < KB2; ++kb)
#pragma unroll
                for (int d = 0; d < NI_MAX; ++d)
                    if (d < ni) {
                        const half8 a = *reinterpret_cast<const half8*>(arow + d * 32 * PITCH + 16 * kb);
                        acc1[d] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, p2f[kb], acc1[d], 0, 0, 0);
                    }
            // Y^T[slab, :] += Z^T[slab, K block] P1[K block, :], hi and lo parts of Z
#pragma unroll
            for (int d = 0; d < NI_MAX; ++d)
#pragma unroll
                for (int kq = 0; kq < 2; ++kq) {
                    const int kk = 2 * (I0 + d) + kq;
                    if (d < ni && (FULL1 || 16 * kk < n1)) {
                        half8 zh, zl;
                        split_hi_lo(acc1[d], 8 * kq, zh, zl);
                        half8 b[A];
#pragma unroll
                        for (int It = 0; It < A; ++It) {
                            if constexpr (P1LDS) b[It] = *reinterpret_cast<const half8*>(&P1s[(It * KB1 + kk) * 64 + l]);
                            else b[It] = p1f[It][kk];
                        }
#pragma unroll
                        for (int It = 0; It < A; ++It) acc2[It] = __builtin_amdgcn_mfma_f32_32x32x16_f16(zh, b[It], acc2[It], 0, 0, 0);
#pragma unroll
                        for (int It = 0; It < A; ++It) acc2[It] = __builtin_amdgcn_mfma_f32_32x32x16_f16(zl, b[It], acc2[It], 0, 0, 0);
                    }
                }
        }

        // ---- per-token absmax: in-lane, DPP over the wave, one float per wave through LDS
        float m = 0.0f;
#pragma unroll
        for (int It = 0; It < A; ++It)
#pragma unroll
            for (int r = 0; r < 16; ++r) m = __builtin_fmaxf(m, __builtin_fabsf(acc2[It][r]));
        m = wave_max(m);
        if (l == 0) red[w] = m;
        __syncthreads();   // (A) every wave is also done reading the token tile
#pragma unroll
        for (int b = 0; b < B; ++b) m = __builtin_fmaxf(m, red[b]);

        const _Float16 sh = (_Float16)(clipv * m * 0.142857149f);   // step = alpha * max / 7, round-to-nearest-even to fp16
        const float s = (float)sh;
        const float inv = (s > 0.0f && s <= 65504.0f) ? __builtin_amdgcn_rcpf(s) : 0.0f;   // 1 ulp: < 1e-6 code units
        const float sl = (inv != 0.0f) ? s : 0.0f;
        const float lim_hi = 7.0f * sl, lim_lo = -8.0f * sl;

        // ---- clamp, round, pack.  fma against 1.5 * 2^23 + 8 leaves code + 8 (0..15) in the low mantissa bits with
        // zeros above up to bit 21, so four results chain with shift-adds and one xor turns offset-binary
        // nibbles into two's complement ones.
#pragma unroll
        for (int It = 0; It < A; ++It) {
            const int ip = 32 * It + c;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint32_t bits[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float yc = __builtin_amdgcn_fmed3f(acc2[It][4 * g + k], lim_lo, lim_hi);
                    bits[k] = __builtin_bit_cast(uint32_t, __builtin_fmaf(yc, inv, 12582920.0f));
                }
                const uint32_t pk = ((((bits[3] << 4) + bits[2]) << 8) + ((bits[1] << 4) + bits[0])) ^ 0x8888u;
                const int jp = 32 * w + 8 * g + 4 * h;
                if (FULL1 || It < A - 1 || ip < n1)
                    *reinterpret_cast<uint16_t*>(stage + ((ip * N2 + jp) >> 1)) = (uint16_t)pk;
            }
        }
        if (have_next) commit(pre_next);
        __syncthreads();   // (B) staged codes and the next tile are visible

        u32x4* dst = reinterpret_cast<u32x4*>(p.out_codes + t * row_bytes_out);
        const int nq = n1 * B;   // 16-byte units of one code row (n1 * N2 / 32)
        for (int q = tid; q < nq; q += NT)
            __builtin_nontemporal_store(reinterpret_cast<const u32x4*>(stage)[q], dst + q);
        if (tid == 0) p.out_scales[t] = sh;
    };

    if constexpr (DEEP) {
        while (true) {
            body(t, pre1, pre0);
            t += G;
            if (t >= p.T) break;
            body(t, pre0, pre1);
            t += G;
            if (t >= p.T) break;
        }
    } else {
        for (; t < p.T; t += G) body(t, pre0, pre0);
    }
}

// ------------------------------------------------------------------------------------
using KernelFn = void (*)(TqDev);

struct Variant {
    KernelFn fn;
    int lds;
};

template <int A, int B>
static Variant variant_ab(bool full1) {
    return full1 ? Variant{&tq_fast_kernel<A, B, true>, FastLds<A, B>::TOTAL}
                 : Variant{&tq_fast_kernel<A, B, false>, FastLds<A, B>::TOTAL};
}

template <int A>
static Variant variant_a(int B, bool full1) {
    switch (B) {
        case 1: return variant_ab<A, 1>(full1);
        case 2: return variant_ab<A, 2>(full1);
        case 3: return variant_ab<A, 3>(full1);
        case 4: return variant_ab<A, 4>(full1);
        case 5: return variant_ab<A, 5>(full1);
        case 6: return variant_ab<A, 6>(full1);
        case 7: return variant_ab<A, 7>(full1);
        default: return variant_ab<A, 8>(full1);
    }
}

static Variant variant(int A, int B, bool full1) {
    switch (A) {
        case 1: return variant_a<1>(B, full1);
        case 2: return variant_a<2>(B, full1);
        case 3: return variant_a<3>(B, full1);
        default: return variant_a<4>(B, full1);
    }
}

bool tq_fast_applicable(const TqDev& d) {
    if (d.n2 % 32 != 0 || !d.vec8 || !d.out_vec16) return false;
    if (reinterpret_cast<uintptr_t>(d.P2) & 15) return false;
    const int n1sq = d.n1 * d.n1;
    const uintptr_t a1 = reinterpret_cast<uintptr_t>(d.P1);
    if ((n1sq & 7) == 0) return (a1 & 15) == 0;
    return (a1 & 3) == 0;
}

int64_t tq_fast_lds_bytes(int n1, int n2) {
    if (n1 < 1 || n1 > kMaxN1 || n2 < 32 || n2 > kMaxN2 || n2 % 32) return 0;
    return variant((n1 + 31) / 32, n2 / 32, n1 % 32 == 0).lds;
}

hipError_t tq_fast_launch(const TqDev& d, hipStream_t stream) {
    const int A = (d.n1 + 31) / 32, B = d.n2 / 32;
    const bool full1 = (d.n1 % 32) == 0;
    const Variant v = variant(A, B, full1);
    const int nt = 64 * B;

    static int wg_per_cu[4][8][2];   // per-variant occupancy, computed once per process (benign race: same value)
    int occ = wg_per_cu[A - 1][B - 1][full1];
    if (occ == 0) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(v.fn), hipFuncAttributeMaxDynamicSharedMemorySize, v.lds);
        if (e != hipSuccess) return e;
        int nb = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, v.fn, nt, v.lds);
        if (e != hipSuccess) return e;
        if (nb < 1) return hipErrorLaunchOutOfResources;
        occ = nb;
        wg_per_cu[A - 1][B - 1][full1] = occ;
    }
    const int cap = env_int("FLATQUANT_WG_PER_CU", 0);
    if (cap > 0 && cap < occ) occ = cap;
    // every workgroup gets the same number of tokens (+-1): grid = ceil(T / ceil(T / resident workgroups))
    const int64_t resident = (int64_t)cu_count() * occ;
    const int64_t rounds = (d.T + resident - 1) / resident;
    const int64_t grid = (d.T + rounds - 1) / rounds;
    hipLaunchKernelGGL(v.fn, dim3((unsigned)grid), dim3(nt), v.lds, stream, d);
    return hipGetLastError();
}

}  // namespace fq
