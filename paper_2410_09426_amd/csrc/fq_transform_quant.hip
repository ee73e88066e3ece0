// Fused per-token Kronecker transform + symmetric INT4 quantization for gfx950.
//
// Computes, for every token row, Q(P1^T X~ P2) (Eq. (2), left factor; the fused
// design of Sec. 3.3 / App. "Detailed Design of Kernel Fusion": both small
// contractions and the quantizer in one launch, intermediates never leave the
// chip).  The mapping to CDNA4 differs from the paper's one-thread-block-per-
// token Triton design:
//
//   * A workgroup has one wavefront per 32-column slab of n2.  Wave w owns
//     output columns j' in [32w, 32w+32).
//   * Contraction over axis 2, Z = X~ P2[:, slab]: MFMA 32x32x16 f16 with the
//     token tile read from LDS as the A operand (rows i, 8 consecutive j per
//     lane = one 16-byte LDS read) and the wave's P2 slab resident in VGPRs as
//     the B operand.  Result: lanes <-> j', registers <-> i.
//   * Contraction over axis 1, Y^T = Z^T P1: the fp32 accumulators of Z are
//     split into fp16 hi + lo parts (so the fp64 oracle's codes are reproduced)
//     and fed straight back as the A operand -- the accumulator layout of one
//     MFMA is a valid A/B operand layout for the next as long as the constant
//     operand (P1) is gathered with the same k-permutation, so there is no LDS
//     round trip.  Result: lanes <-> i', registers <-> j' with 4 consecutive j'
//     per register quad, i.e. 4 consecutive channels = 2 packed bytes per lane.
//   * absmax: in-lane over registers, wave butterfly, one float per wave in LDS.
//   * Codes are staged in LDS in channel order and written with 16-byte stores.
//   * Workgroups are persistent over tokens; the next token row is prefetched
//     into registers while the current one is in the MFMA pipe.
#include "fq_internal.h"

namespace fq {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));


__device__ __forceinline__ half8 split_hi(const float* z, float* resid) {
    // hi = fp16(z) rounded toward zero (never overflows to inf), resid = z - hi exactly
    half8 h;
#pragma unroll
    for (int k = 0; k < 8; k += 2) {
        auto pk = __builtin_amdgcn_cvt_pkrtz(z[k], z[k + 1]);
        h[k] = (_Float16)pk[0];
        h[k + 1] = (_Float16)pk[1];
        resid[k] = z[k] - (float)h[k];
        resid[k + 1] = z[k + 1] - (float)h[k + 1];
    }
    return h;
}

__device__ __forceinline__ half8 to_half8_rtz(const float* z) {
    half8 h;
#pragma unroll
    for (int k = 0; k < 8; k += 2) {
        auto pk = __builtin_amdgcn_cvt_pkrtz(z[k], z[k + 1]);
        h[k] = (_Float16)pk[0];
        h[k + 1] = (_Float16)pk[1];
    }
    return h;
}

// round-half-even of a value already clamped to [-8, 7], as a 4-bit two's complement nibble
__device__ __forceinline__ uint32_t nibble(float y, float inv) {
    float u = __builtin_fminf(__builtin_fmaxf(y * inv, -8.0f), 7.0f);
    return (uint32_t)(int)__builtin_rintf(u) & 0xFu;
}

// MX: MXFP4 output for the shapes the specialised kernels do not take (n2 not a multiple of 32, where a block of 32
// consecutive channels straddles rows of X~ and column slabs): the token's Y is staged in LDS as fp32 in channel order,
// then one thread per block takes its 32 values, forms the shared exponent and converts.
template <int A, int B, bool P1LDS, bool MX = false>
__global__ __launch_bounds__(64 * B) void tq_kernel(TqDev p) {
    constexpr int NT = 64 * B;
    constexpr int PITCH = 32 * B + kLdsPad;      // halves per LDS row of the token tile
    constexpr int XS_HALVES = 32 * A * PITCH;
    constexpr int STAGE_BYTES = (MX ? 4096 : 512) * A * B;     // >= n / 2 bytes of codes, or 4 n bytes of fp32 values
    constexpr int NPRE = 2 * A;                  // 16-byte chunks per thread per token (upper bound)
    constexpr int KB2 = 2 * B;                   // K blocks (of 16) over j
    constexpr int KB1 = 2 * A;                   // K blocks (of 16) over i

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    _Float16* Xs = reinterpret_cast<_Float16*>(smem);
    uint8_t* stage = smem + XS_HALVES * 2;
    float* red = reinterpret_cast<float*>(stage + STAGE_BYTES);
    u32x4* P1s = reinterpret_cast<u32x4*>(red + 8);

    const int tid = threadIdx.x;
    const int l = tid & 63, w = tid >> 6, c = l & 31, h = l >> 5;
    const int n1 = p.n1, n2 = p.n2;
    const int n = n1 * n2;

    // ---- one-off: zero the tile (pad rows/columns stay zero for the whole kernel)
    for (int q = tid; q < XS_HALVES / 8; q += NT) reinterpret_cast<u32x4*>(Xs)[q] = u32x4{0u, 0u, 0u, 0u};

    // ---- one-off: this wave's P2 slab as B-operand fragments (lane <-> j', 8 k-values <-> j)
    half8 p2f[KB2];
#pragma unroll
    for (int kb = 0; kb < KB2; ++kb) {
        const int jp = 32 * w + c;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const int j = 16 * kb + 8 * h + s;
            p2f[kb][s] = (j < n2 && jp < n2) ? (p.P2 ? p.P2[j * n2 + jp] : (_Float16)(j == jp ? 1.0f : 0.0f)) : (_Float16)0;
        }
    }
    // ---- one-off: P1 as B-operand fragments of the second contraction (lane <-> i'),
    // gathered with the k-permutation that the accumulator layout of the first one imposes:
    // K block kk, slot s of half-wave h  <->  i = 32(kk/2) + 8(2(kk%2) + s/4) + 4h + s%4.
    half8 p1f[P1LDS ? 1 : A][P1LDS ? 1 : KB1];
    if constexpr (P1LDS) {
        for (int e = tid; e < A * KB1 * 64; e += NT) {
            const int ln = e & 63, kk = (e >> 6) % KB1, It = (e >> 6) / KB1;
            const int cc = ln & 31, hh = ln >> 5;
            const int ip = 32 * It + cc;
            half8 f;
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const int i = 32 * (kk >> 1) + 8 * (2 * (kk & 1) + (s >> 2)) + 4 * hh + (s & 3);
                f[s] = (i < n1 && ip < n1) ? (p.P1 ? p.P1[i * n1 + ip] : (_Float16)(i == ip ? 1.0f : 0.0f)) : (_Float16)0;
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
                    p1f[It][kk][s] = (i < n1 && ip < n1) ? (p.P1 ? p.P1[i * n1 + ip] : (_Float16)(i == ip ? 1.0f : 0.0f)) : (_Float16)0;
                }
            }
    }

    // ---- per-thread LDS destinations of the 16-byte chunks of a token row (fixed for all tokens)
    const int nchunks = n >> 3;
    int xoff[NPRE];
#pragma unroll
    for (int k = 0; k < NPRE; ++k) {
        const int q = tid + k * NT;
        const int e = q * 8;
        const int i = e / n2;
        xoff[k] = (p.vec8 && q < nchunks) ? i * PITCH + (e - i * n2) : -1;
    }

    auto issue = [&](int64_t t, u32x4 (&pre)[NPRE]) {
        const u32x4* src = reinterpret_cast<const u32x4*>(p.x + t * p.x_stride);
#pragma unroll
        for (int k = 0; k < NPRE; ++k)
            if (xoff[k] >= 0) pre[k] = __builtin_nontemporal_load(src + tid + k * NT);
    };
    auto commit = [&](const u32x4 (&pre)[NPRE]) {
#pragma unroll
        for (int k = 0; k < NPRE; ++k)
            if (xoff[k] >= 0) *reinterpret_cast<u32x4*>(Xs + xoff[k]) = pre[k];
    };
    // rows that cannot move in 16-byte chunks (n2 not a multiple of 8, or an unaligned x): pairs of halves, requested
    // into registers before the MFMA work like the chunks above (n / 2 pairs over the workgroup: at most 8 A per thread);
    // a pair never straddles a row (n2 is even), and its row is umulhi(2 u, magic) with the magic divisor from the host
    constexpr int NPS = 8 * A;
    uint32_t pres[NPS];
    auto issue_slow = [&](int64_t t) {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(p.x + t * p.x_stride);
#pragma unroll
        for (int k = 0; k < NPS; ++k) {
            const int u = tid + k * NT;
            if (u < (n >> 1)) pres[k] = src[u];
        }
    };
    auto commit_slow = [&]() {
#pragma unroll
        for (int k = 0; k < NPS; ++k) {
            const int u = tid + k * NT;
            if (u < (n >> 1)) {
                const int e = 2 * u, i = (int)__umulhi((uint32_t)e, p.n2_magic);
                *reinterpret_cast<uint32_t*>(Xs + i * PITCH + (e - i * n2)) = pres[k];
            }
        }
    };

    __syncthreads();   // zero fill (and P1s) complete before the first tile lands
    u32x4 pre[NPRE];
    int64_t t = blockIdx.x;
    if (t < p.T) {
        if (p.vec8) { issue(t, pre); commit(pre); } else { issue_slow(t); commit_slow(); }
    }
    __syncthreads();

    for (; t < p.T; t += gridDim.x) {
        const int64_t tn = t + gridDim.x;
        const bool have_next = tn < p.T;
        if (have_next) {
            if (p.vec8) issue(tn, pre); else issue_slow(tn);
        }

        f32x16 acc2[A];
#pragma unroll
        for (int It = 0; It < A; ++It)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc2[It][r] = 0.0f;

#pragma unroll
        for (int I = 0; I < A; ++I) {
            // Z[32I .. 32I+31, slab] = X~[32I.., :] P2[:, slab]
            f32x16 acc1;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc1[r] = 0.0f;
            const _Float16* arow = Xs + (32 * I + c) * PITCH + 8 * h;
#pragma unroll
            for (int kb = 0; kb < KB2; ++kb) {
                if (16 * kb < n2) {
                    const half8 a = *reinterpret_cast<const half8*>(arow + 16 * kb);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, p2f[kb], acc1, 0, 0, 0);
                }
            }
            // Y^T[slab, :] += Z^T[slab, K block] P1[K block, :], hi and lo parts of Z
#pragma unroll
            for (int kq = 0; kq < 2; ++kq) {
                const int kk = 2 * I + kq;
                if (16 * kk < n1) {
                    float z[8], resid[8];
#pragma unroll
                    for (int s = 0; s < 8; ++s) z[s] = acc1[8 * kq + s];
                    const half8 zh = split_hi(z, resid);
                    const half8 zl = to_half8_rtz(resid);
#pragma unroll
                    for (int It = 0; It < A; ++It) {
                        half8 b;
                        if constexpr (P1LDS) b = *reinterpret_cast<const half8*>(&P1s[(It * KB1 + kk) * 64 + l]);
                        else b = p1f[It][kk];
                        acc2[It] = __builtin_amdgcn_mfma_f32_32x32x16_f16(zh, b, acc2[It], 0, 0, 0);
                        acc2[It] = __builtin_amdgcn_mfma_f32_32x32x16_f16(zl, b, acc2[It], 0, 0, 0);
                    }
                }
            }
        }

        const float clipv = p.clip[p.clip_mode ? t : 0];
        _Float16 sh = (_Float16)0.0f;
        if constexpr (MX) {
            __syncthreads();   // (A) all waves are done reading the token tile
            float* stagef = reinterpret_cast<float*>(stage);
#pragma unroll
            for (int It = 0; It < A; ++It) {
                const int ip = 32 * It + c;
#pragma unroll
                for (int g = 0; g < 4; ++g)
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const int jp = 32 * w + 8 * g + 4 * h + k;
                        if (ip < n1 && jp < n2) stagef[ip * n2 + jp] = acc2[It][4 * g + k];
                    }
            }
        } else {
        // ---- per-token absmax (padded rows/columns are exact zeros)
        float m = 0.0f;
#pragma unroll
        for (int It = 0; It < A; ++It)
#pragma unroll
            for (int r = 0; r < 16; ++r) m = __builtin_fmaxf(m, __builtin_fabsf(acc2[It][r]));
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) m = __builtin_fmaxf(m, __shfl_xor(m, off));
        if (l == 0) red[w] = m;
        __syncthreads();   // (A) all waves are also done reading the token tile
#pragma unroll
        for (int b = 0; b < B; ++b) m = __builtin_fmaxf(m, red[b]);

        sh = (_Float16)(clipv * m / 7.0f);   // round-to-nearest-even to fp16
        const float s = (float)sh;
        const float inv = (s > 0.0f && s <= 65504.0f) ? 1.0f / s : 0.0f;

        // ---- round, clamp, pack 4 consecutive channels per register quad, stage in channel order
#pragma unroll
        for (int It = 0; It < A; ++It) {
            const int ip = 32 * It + c;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int jp = 32 * w + 8 * g + 4 * h;
                if (ip < n1 && jp < n2) {
                    const uint32_t pk = nibble(acc2[It][4 * g + 0], inv) | (nibble(acc2[It][4 * g + 1], inv) << 4) |
                                        (nibble(acc2[It][4 * g + 2], inv) << 8) | (nibble(acc2[It][4 * g + 3], inv) << 12);
                    const int byte = (ip * n2 + jp) >> 1;
                    if ((n2 & 3) == 0) {
                        *reinterpret_cast<uint16_t*>(stage + byte) = (uint16_t)pk;
                    } else {
                        stage[byte] = (uint8_t)pk;
                        if (jp + 2 < n2) stage[byte + 1] = (uint8_t)(pk >> 8);
                    }
                }
            }
        }
        }
        // ---- next token tile into LDS (its loads were issued before the MFMA work)
        if (have_next) {
            if (p.vec8) commit(pre); else commit_slow();
        }
        __syncthreads();   // (B) staged codes and next tile visible

        uint8_t* dst = p.out_codes + t * (int64_t)(n >> 1);
        if constexpr (MX) {
            // Block b = channels 32 b .. 32 b + 31: exponent floor(log2(alpha max)) - 2 (0 for an all-zero block), elements
            // converted with the stored exponent (the conversion reads the exponent field of its scale operand only,
            // and field 0 means 2^-127); 16 bytes of codes per block, exponents row-major or in the product's tile order
            const float* stagef = reinterpret_cast<const float*>(stage);
            uint8_t* exps = reinterpret_cast<uint8_t*>(p.out_scales);
            const int nblk = n >> 5;
            for (int b = tid; b < nblk; b += NT) {
                float y[32];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const float4 v = reinterpret_cast<const float4*>(stagef + 32 * b)[k];
                    y[4 * k] = v.x; y[4 * k + 1] = v.y; y[4 * k + 2] = v.z; y[4 * k + 3] = v.w;
                }
                float bm = 0.0f;
#pragma unroll
                for (int k = 0; k < 32; ++k) bm = __builtin_fmaxf(bm, __builtin_fabsf(y[k]));
                bm *= clipv;
                const uint32_t be = (__builtin_bit_cast(uint32_t, bm) >> 23) & 0xffu;
                const uint32_t e = be > 2 ? be - 2 : 0;
                const float scale = __builtin_bit_cast(float, e << 23);
                u32x4 o;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    uint32_t pk = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(0u, y[8 * d], y[8 * d + 1], scale, 0);
                    pk = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(pk, y[8 * d + 2], y[8 * d + 3], scale, 1);
                    pk = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(pk, y[8 * d + 4], y[8 * d + 5], scale, 2);
                    pk = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(pk, y[8 * d + 6], y[8 * d + 7], scale, 3);
                    o[d] = pk;
                }
                reinterpret_cast<u32x4*>(dst)[b] = o;
                if (p.mx_tiled) exps[((((t >> 7) * (int64_t)(n >> 8) + (b >> 3)) * 128 + (t & 127)) << 3) + (b & 7)] = (uint8_t)e;
                else exps[t * (int64_t)nblk + b] = (uint8_t)e;
            }
        } else {
            if (p.out_vec16) {
                for (int q = tid; q < (n >> 5); q += NT)
                    __builtin_nontemporal_store(reinterpret_cast<const u32x4*>(stage)[q], reinterpret_cast<u32x4*>(dst) + q);
            } else {
                for (int q = tid; q < (n >> 1); q += NT) dst[q] = stage[q];
            }
            if (tid == 0) p.out_scales[t] = sh;
        }
    }
}

// ------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------
using KernelFn = void (*)(TqDev);

template <int A, int B>
static constexpr KernelFn kernel_for() { return &tq_kernel<A, B, (A >= 3)>; }

static KernelFn kernel_table(int A, int B) {
    static const KernelFn tab[4][8] = {
        {kernel_for<1, 1>(), kernel_for<1, 2>(), kernel_for<1, 3>(), kernel_for<1, 4>(), kernel_for<1, 5>(), kernel_for<1, 6>(), kernel_for<1, 7>(), kernel_for<1, 8>()},
        {kernel_for<2, 1>(), kernel_for<2, 2>(), kernel_for<2, 3>(), kernel_for<2, 4>(), kernel_for<2, 5>(), kernel_for<2, 6>(), kernel_for<2, 7>(), kernel_for<2, 8>()},
        {kernel_for<3, 1>(), kernel_for<3, 2>(), kernel_for<3, 3>(), kernel_for<3, 4>(), kernel_for<3, 5>(), kernel_for<3, 6>(), kernel_for<3, 7>(), kernel_for<3, 8>()},
        {kernel_for<4, 1>(), kernel_for<4, 2>(), kernel_for<4, 3>(), kernel_for<4, 4>(), kernel_for<4, 5>(), kernel_for<4, 6>(), kernel_for<4, 7>(), kernel_for<4, 8>()},
    };
    return tab[A - 1][B - 1];
}

template <int A, int B>
static constexpr KernelFn mx_kernel_for() { return &tq_kernel<A, B, (A >= 3), true>; }

static KernelFn mx_kernel_table(int A, int B) {
    static const KernelFn tab[4][8] = {
        {mx_kernel_for<1, 1>(), mx_kernel_for<1, 2>(), mx_kernel_for<1, 3>(), mx_kernel_for<1, 4>(), mx_kernel_for<1, 5>(), mx_kernel_for<1, 6>(), mx_kernel_for<1, 7>(), mx_kernel_for<1, 8>()},
        {mx_kernel_for<2, 1>(), mx_kernel_for<2, 2>(), mx_kernel_for<2, 3>(), mx_kernel_for<2, 4>(), mx_kernel_for<2, 5>(), mx_kernel_for<2, 6>(), mx_kernel_for<2, 7>(), mx_kernel_for<2, 8>()},
        {mx_kernel_for<3, 1>(), mx_kernel_for<3, 2>(), mx_kernel_for<3, 3>(), mx_kernel_for<3, 4>(), mx_kernel_for<3, 5>(), mx_kernel_for<3, 6>(), mx_kernel_for<3, 7>(), mx_kernel_for<3, 8>()},
        {mx_kernel_for<4, 1>(), mx_kernel_for<4, 2>(), mx_kernel_for<4, 3>(), mx_kernel_for<4, 4>(), mx_kernel_for<4, 5>(), mx_kernel_for<4, 6>(), mx_kernel_for<4, 7>(), mx_kernel_for<4, 8>()},
    };
    return tab[A - 1][B - 1];
}

bool tq_supported(int n1, int n2) {
    return n1 >= 1 && n1 <= kMaxN1 && n2 >= 2 && n2 <= kMaxN2 && (n2 % 2) == 0;
}

static int64_t generic_lds_bytes(int n1, int n2) {
    const int A = (n1 + 31) / 32, B = (n2 + 31) / 32;
    int64_t b = (int64_t)32 * A * (32 * B + kLdsPad) * 2 + 512 * A * B + 32;
    if (A >= 3) b += (int64_t)A * 2 * A * 64 * 16;
    return b;
}

int64_t tq_lds_bytes(int n1, int n2) {
    if (!tq_supported(n1, n2)) return 0;
    const int64_t b = generic_lds_bytes(n1, n2);
    const int64_t f = tq_fast_lds_bytes(n1, n2);   // the specialised kernels stage P1/P2 in LDS as well
    return f > b ? f : b;
}

static int64_t generic_mx_lds_bytes(int n1, int n2) {
    const int A = (n1 + 31) / 32, B = (n2 + 31) / 32;
    return generic_lds_bytes(n1, n2) + (int64_t)(4096 - 512) * A * B;
}

// MXFP4 output through the general kernel: any supported (n1, n2) with whole blocks of 32 channels per row whose
// fp32 staging fits in LDS beside the token tile (64 x 172: 74 KB), 16-byte aligned code rows.
bool tq_mx_generic_applicable(const TqDev& d) {
    const int64_t n = (int64_t)d.n1 * d.n2;
    return tq_supported(d.n1, d.n2) && n % 32 == 0 && d.out_vec16 && d.P1 && d.P2 && generic_mx_lds_bytes(d.n1, d.n2) <= 160 * 1024;
}

hipError_t tq_mx_generic_launch(const TqDev& d, hipStream_t stream) {
    const int A = (d.n1 + 31) / 32, B = (d.n2 + 31) / 32;
    KernelFn fn = mx_kernel_table(A, B);
    const int lds = (int)generic_mx_lds_bytes(d.n1, d.n2);
    static OccCache occ_cache[4][8];
    int occ = 0;
    {
        hipError_t e = kernel_occupancy(reinterpret_cast<const void*>(fn), 64 * B, lds, occ_cache[A - 1][B - 1], occ);
        if (e != hipSuccess) return e;
    }
    int64_t grid = (int64_t)cu_count() * occ;
    if (grid > d.T) grid = d.T;
    return launch(fn, dim3((unsigned)grid), dim3(64 * B), lds, stream, d);
}

TqDev tq_dev_args(const TqArgs& a) {
    TqDev d;
    d.x = a.x; d.P1 = a.P1; d.P2 = a.P2; d.clip = a.clip;
    d.out_codes = a.out_codes; d.out_scales = a.out_scales;
    d.x_stride = a.x_stride; d.T = a.T; d.n1 = a.n1; d.n2 = a.n2; d.clip_mode = a.clip_mode;
    d.mx_tiled = a.mx_tiled;
    d.n1_magic = a.n1 >= 2 ? (uint32_t)(0x100000000ull / (uint64_t)a.n1) + 1u : 0u;
    d.n2_magic = a.n2 >= 2 ? (uint32_t)(0x100000000ull / (uint64_t)a.n2) + 1u : 0u;
    d.vec8 = (a.n2 % 8 == 0) && (a.x_stride % 8 == 0) && ((reinterpret_cast<uintptr_t>(a.x) & 15) == 0);
    const int64_t n = (int64_t)a.n1 * a.n2;
    d.out_vec16 = (n % 32 == 0) && ((reinterpret_cast<uintptr_t>(a.out_codes) & 15) == 0);
    return d;
}

hipError_t tq_launch(const TqArgs& a, hipStream_t stream) {
    const int A = (a.n1 + 31) / 32, B = (a.n2 + 31) / 32;
    KernelFn fn = kernel_table(A, B);
    const int lds = (int)generic_lds_bytes(a.n1, a.n2);
    const int nt = 64 * B;

    const TqDev d = tq_dev_args(a);
    // FLATQUANT_FORCE_GENERIC=1 keeps the general kernel testable on shapes the specialised ones would take
    if (tq_fast_applicable(d) && env_int("FLATQUANT_FORCE_GENERIC", 0) == 0) return tq_fast_launch(d, stream);

    static OccCache occ_cache[4][8];   // per variant and device
    int occ = 0;
    {
        hipError_t e = kernel_occupancy(reinterpret_cast<const void*>(fn), nt, (int)lds, occ_cache[A - 1][B - 1], occ);
        if (e != hipSuccess) return e;
    }
    const int cap = env_int("FLATQUANT_WG_PER_CU", 0);
    if (cap > 0 && cap < occ) occ = cap;
    int64_t grid = (int64_t)cu_count() * occ;
    if (grid > a.T) grid = a.T;

    return launch(fn, dim3((unsigned)grid), dim3(nt), lds, stream, d);
}

}  // namespace fq
