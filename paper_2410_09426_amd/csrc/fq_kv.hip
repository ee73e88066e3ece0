// KV-cache variant for gfx950: per-head dense transform + group-wise asymmetric INT4.
//
// For every (token, head) group of D = 128 values: y = kv_g P_h (Sec. 3.2
// "Self-Attention": P_h / P_v are applied head by head and are not decomposed),
// then asymmetric INT4 with one step and one zero point per group (Sec. 4.1
// "Quantization": group size 128 = head_dim).
//
// Mapping: blockIdx.y is the head, so every wave of a workgroup shares one P_h,
// kept in LDS as ready-made MFMA A-operand fragments.  A wave takes 32 tokens:
//   Y^T[d', token] = sum_d P_h[d, d'] kv[token, d]
// with M = d' (4 tiles of 32), N = 32 tokens, K = d (8 blocks of 16).  The B
// operand comes straight from global memory (lane <-> token, 16 bytes <-> 8
// consecutive d).  In the result a lane holds, for its token, 64 of the 128
// outputs (the other half-wave holds the rest) in runs of 4 consecutive d', so
// min/max need one cross-half exchange and 4 codes pack into 2 bytes in-lane.
#include "fq_internal.h"

namespace fq {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int KV_D = 128;
constexpr int KV_WAVES = 4;
constexpr int KV_TOK_PER_WAVE = 32;
constexpr int KV_STAGE_PITCH = 80;   // bytes per staged code row (64 + pad)

struct KvDev {
    const _Float16* kv;
    const _Float16* P;
    uint8_t* out_codes;
    _Float16* out_scales;
    _Float16* out_zeros;
    int64_t T;
    int H, Hp;
    float clip;
};

__global__ __launch_bounds__(64 * KV_WAVES) void kv_kernel(KvDev p) {
    constexpr int MT = KV_D / 32;   // 4 tiles over d'
    constexpr int KB = KV_D / 16;   // 8 K blocks over d
    __shared__ __attribute__((aligned(16))) uint4 Pf[MT * KB * 64];                       // 32 KB of A fragments
    __shared__ __attribute__((aligned(16))) uint8_t stage[KV_WAVES][32 * KV_STAGE_PITCH];  // per-wave code rows

    const int tid = threadIdx.x;
    const int l = tid & 63, w = tid >> 6, c = l & 31, h = l >> 5;
    const int head = blockIdx.y;
    const _Float16* Ph = p.P + (size_t)(p.Hp == 1 ? 0 : head) * KV_D * KV_D;

    // A fragment (M tile mt, K block kb): lane (c, h) holds P_h[16kb + 8h + s][32mt + c], s = 0..7
    for (int e = tid; e < MT * KB * 64; e += 64 * KV_WAVES) {
        const int ln = e & 63, kb = (e >> 6) % KB, mt = (e >> 6) / KB;
        const int cc = ln & 31, hh = ln >> 5;
        half8 f;
#pragma unroll
        for (int s = 0; s < 8; ++s) f[s] = Ph[(16 * kb + 8 * hh + s) * KV_D + 32 * mt + cc];
        *reinterpret_cast<half8*>(&Pf[e]) = f;
    }
    __syncthreads();

    const int64_t nblk = (p.T + KV_TOK_PER_WAVE - 1) / KV_TOK_PER_WAVE;   // 32-token blocks
    for (int64_t blk = (int64_t)blockIdx.x * KV_WAVES + w; blk < nblk; blk += (int64_t)gridDim.x * KV_WAVES) {
        const int64_t tok = blk * KV_TOK_PER_WAVE + c;
        const bool live = tok < p.T;
        const int64_t grp = (live ? tok : p.T - 1) * p.H + head;          // clamp: dead lanes re-read the last token
        const uint4* row = reinterpret_cast<const uint4*>(p.kv + grp * KV_D);

        half8 bf[KB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            uint4 v = row[2 * kb + h];
            bf[kb] = *reinterpret_cast<half8*>(&v);
        }
        f32x16 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][r] = 0.0f;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                const half8 a = *reinterpret_cast<const half8*>(&Pf[(mt * KB + kb) * 64 + l]);
                acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, bf[kb], acc[mt], 0, 0, 0);
            }
        }
        // group range: in-lane over 64 values, then the other half-wave's 64
        float mx = 0.0f, mn = 0.0f;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                mx = __builtin_fmaxf(mx, acc[mt][r]);
                mn = __builtin_fminf(mn, acc[mt][r]);
            }
        mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32));
        mn = __builtin_fminf(mn, __shfl_xor(mn, 32));
        mx *= p.clip;
        mn *= p.clip;
        const _Float16 sh = (_Float16)((mx - mn) / 15.0f);
        const float s = (float)sh;
        const float inv = (s > 0.0f && s <= 65504.0f) ? 1.0f / s : 0.0f;
        const float z = __builtin_fminf(__builtin_fmaxf(__builtin_rintf(-mn * inv), 0.0f), 15.0f);

        uint8_t* srow = &stage[w][c * KV_STAGE_PITCH];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint32_t pk = 0;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float q = __builtin_fminf(__builtin_fmaxf(__builtin_rintf(acc[mt][4 * g + k] * inv) + z, 0.0f), 15.0f);
                    pk |= (uint32_t)(int)q << (4 * k);
                }
                const int dp = 32 * mt + 8 * g + 4 * h;   // first of 4 consecutive output channels
                *reinterpret_cast<uint16_t*>(srow + (dp >> 1)) = (uint16_t)pk;
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // 32 rows x 64 bytes: lane -> (row l/4 + 16k, 16-byte chunk l%4)
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int r = (l >> 2) + 16 * k, ch = l & 3;
            const int64_t tk = blk * KV_TOK_PER_WAVE + r;
            if (tk < p.T) {
                const uint4 v = *reinterpret_cast<const uint4*>(&stage[w][r * KV_STAGE_PITCH + 16 * ch]);
                *reinterpret_cast<uint4*>(p.out_codes + (tk * p.H + head) * (KV_D / 2) + 16 * ch) = v;
            }
        }
        if (live && h == 0) {
            p.out_scales[grp] = sh;
            p.out_zeros[grp] = (_Float16)z;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();   // staged rows are consumed before the next block overwrites them
    }
}

hipError_t kv_launch(const KvArgs& a, hipStream_t stream) {
    const int64_t nblk = (a.T + KV_TOK_PER_WAVE - 1) / KV_TOK_PER_WAVE;
    int64_t gx = (nblk + KV_WAVES - 1) / KV_WAVES;
    const int64_t cap = (int64_t)cu_count() * 2 * 8 / (a.H < 8 ? a.H : 8) + 1;   // about 2 workgroups per CU in total
    const int wg_cap = env_int("FLATQUANT_KV_GRID_X", 0);
    if (gx > cap) gx = cap;
    if (wg_cap > 0 && gx > wg_cap) gx = wg_cap;
    KvDev d;
    d.kv = a.kv; d.P = a.P; d.out_codes = a.out_codes; d.out_scales = a.out_scales; d.out_zeros = a.out_zeros;
    d.T = a.T; d.H = a.H; d.Hp = a.Hp; d.clip = a.clip;
    hipLaunchKernelGGL(kv_kernel, dim3((unsigned)gx, (unsigned)a.H), dim3(64 * KV_WAVES), 0, stream, d);
    return hipGetLastError();
}

}  // namespace fq
