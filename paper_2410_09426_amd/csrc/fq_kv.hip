// KV-cache variant for gfx950: per-head dense transform + group-wise asymmetric b-bit codes.
//
// For every (token, head) group of D = 128 values: y = kv_g P_h (Sec. 3.2
// "Self-Attention": P_h / P_v are applied head by head and are not decomposed),
// then asymmetric quantization with one step and one zero point per group (Sec. 4.1
// "Quantization": group size 128 = head_dim, 4 bits; App. "KV Cache Quantization":
// the same grid with 3 and 2 bits).
//
// Mapping: blockIdx.y is the head, so every wave of a workgroup shares one P_h.
// P_h is fetched once per workgroup with coalesced 16-byte loads and re-laid in
// LDS as ready-made MFMA A-operand fragments.  Workgroups are persistent; a wave
// takes 32 tokens at a time:
//   Y^T[d', token] = sum_d P_h[d, d'] kv[token, d]
// with M = d' (4 tiles of 32), N = 32 tokens, K = d (8 blocks of 16).  The B
// operand comes straight from global memory (lane <-> token, 16 bytes <-> 8
// consecutive d) and the next 32 tokens are prefetched into registers while the
// current ones are in the MFMA pipe.  In the result a lane holds, for its token,
// 64 of the 128 outputs (the other half-wave holds the rest).  The M index of a
// 32-row tile is mapped to d' with its 4-row chunks 1 and 2 swapped (a free choice
// when the fragments are built), which turns the accumulator layout's runs of 4
// into runs of 8 consecutive d': 8 codes pack into 4, 3 or 2 whole bytes in-lane.
// min/max need one cross-half exchange.  Packed rows are staged per wave in LDS
// and leave with 16-byte stores.
#include "fq_internal.h"
#include "fq_device.h"

namespace fq {

constexpr int KV_D = 128;
constexpr int KV_WAVES = 4;
constexpr int KV_NT = 64 * KV_WAVES;
constexpr int KV_TOK = 32;                 // tokens per wave per step
constexpr int KV_STAGE_PITCH = 80;         // bytes per staged code row (up to 64 + pad)
constexpr int KV_MT = KV_D / 32;           // 4 tiles over d'
constexpr int KV_KB = KV_D / 16;           // 8 K blocks over d
constexpr int KV_FRAG_BYTES = KV_MT * KV_KB * 64 * 16;        // 32 KB of A fragments
constexpr int KV_FLAT_ROWS = KV_D;                            // rows of P_h staged per pass (all of them: one workgroup per CU has the LDS)
constexpr int KV_PASSES = KV_D / KV_FLAT_ROWS;
constexpr int KV_FLAT_BYTES = KV_FLAT_ROWS * (KV_D + 8) * 2;  // row-major, padded pitch, while fragments are built
constexpr int KV_STAGE_BYTES = KV_WAVES * 32 * KV_STAGE_PITCH;
constexpr int KV_LDS_BYTES = KV_FRAG_BYTES + (KV_FLAT_BYTES > KV_STAGE_BYTES ? KV_FLAT_BYTES : KV_STAGE_BYTES);
// transform-only mode (fp16 out): the staged rows are 256 bytes wide
constexpr int KV_OUT_PITCH = 2 * KV_D + 16;
constexpr int KV_OUT_STAGE_BYTES = KV_WAVES * 32 * KV_OUT_PITCH;
constexpr int KV_OUT_LDS_BYTES = KV_FRAG_BYTES + (KV_FLAT_BYTES > KV_OUT_STAGE_BYTES ? KV_FLAT_BYTES : KV_OUT_STAGE_BYTES);

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

// BITS = 2, 3, 4: asymmetric codes of that width + step + zero point per group.  BITS = 0: the transformed rows
// themselves, rounded to fp16 (p.out_codes then points at an fp16 [T, H, D] tensor): the query side of a transformed
// key cache.
template <int BITS>
__global__ __launch_bounds__(KV_NT) __attribute__((amdgpu_waves_per_eu(2))) void kv_kernel(KvDev p) {
    constexpr bool QUANT = BITS != 0;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    u32x4* Pf = reinterpret_cast<u32x4*>(smem);                               // fragment table
    _Float16* Pflat = reinterpret_cast<_Float16*>(smem + KV_FRAG_BYTES);      // prologue only
    uint8_t* stage_all = smem + KV_FRAG_BYTES;                                // loop only (reuses Pflat's space)

    const int tid = threadIdx.x;
    const int l = tid & 63, c = l & 31, h = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: block indices and base addresses stay scalar
    const int head = blockIdx.y;
    const _Float16* Ph = p.P + (size_t)(p.Hp == 1 ? 0 : head) * KV_D * KV_D;
    const int64_t nblk = (p.T + KV_TOK - 1) / KV_TOK;
    const int64_t bstep = (int64_t)gridDim.x * KV_WAVES;

    // Group (token, head) addressing.  Block `blk` starts at group blk * 32 * H + head (scalar); a lane adds the offset
    // of its token, r tokens further on.  Tokens past the end are clamped to the last one: such lanes re-read its row
    // and later store its (identical) results onto it, so no access needs a branch.
    auto first_group = [&](int64_t blk) { return blk * KV_TOK * p.H + head; };
    auto group_ofs = [&](int64_t blk, int r) -> uint32_t {
        const int64_t left = p.T - 1 - blk * KV_TOK;                       // scalar
        const int rem = left < KV_TOK - 1 ? (int)left : KV_TOK - 1;
        return (uint32_t)((r < rem ? r : rem) * p.H);
    };
    auto issue = [&](int64_t blk, u32x4 (&r)[KV_KB]) {
        const int64_t b = blk < nblk ? blk : nblk - 1;
        const u32x4* row = reinterpret_cast<const u32x4*>(p.kv + first_group(b) * KV_D) + (size_t)group_ofs(b, c) * (KV_D / 8);
#pragma unroll
        for (int kb = 0; kb < KV_KB; ++kb) r[kb] = row[2 * kb + h];   // cached: a 128-byte line is shared by 4 of these loads
    };

    int64_t blk = (int64_t)blockIdx.x * KV_WAVES + w;
    u32x4 cur[KV_KB], nxt[KV_KB];

    // ---- P_h: coalesced loads -> LDS (padded pitch) -> A fragments: lane (c, h) of fragment (mt, kb) holds
    // P_h[16kb + 8h + s][32mt + c'], s = 0..7, c' = c with its 4-column chunks 1 and 2 (of each 16) exchanged.  The LDS copy is made in KV_PASSES passes, but
    // all of P_h is requested up front, and the first token rows only once it has arrived.  A CU's vector memory pipe
    // returns data in request order: if the workgroups that start first queued their rows (HBM) at once, the P_h
    // requests (L2) of the workgroups that start a little later on the same CU would wait behind them for microseconds,
    // and those workgroups would end the kernel late (measured: 11 us to build the fragments instead of 3).
    constexpr int CH = KV_FLAT_ROWS * KV_D / 8;   // chunks of 16 bytes per pass
    u32x4 v[KV_PASSES][CH / KV_NT];
#pragma unroll
    for (int pass = 0; pass < KV_PASSES; ++pass)
#pragma unroll
        for (int k = 0; k < CH / KV_NT; ++k) v[pass][k] = reinterpret_cast<const u32x4*>(Ph)[pass * CH + tid + k * KV_NT];
#pragma unroll
    for (int pass = 0; pass < KV_PASSES; ++pass) {
        if (pass > 0) __syncthreads();   // previous pass fully consumed
#pragma unroll
        for (int k = 0; k < CH / KV_NT; ++k) {
            const int q = tid + k * KV_NT, r = q >> 4, cc = q & 15;
            *reinterpret_cast<u32x4*>(Pflat + r * (KV_D + 8) + cc * 8) = v[pass][k];
        }
        if (pass == KV_PASSES - 1) {   // all of P_h has arrived: only now request the first token rows (see above)
            __builtin_amdgcn_sched_barrier(0);
            issue(blk, cur);
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
        for (int e = tid; e < KV_MT * (KV_KB / KV_PASSES) * 64; e += KV_NT) {
            const int ln = e & 63, kbl = (e >> 6) % (KV_KB / KV_PASSES), mt = (e >> 6) / (KV_KB / KV_PASSES);
            const int cc = ln & 31, hh = ln >> 5;
            // e % 64 is the lane, so whole 16-lane blocks cooperate in the transposing reads
            const half8 f = lds_column8<true>(Pflat, KV_D + 8, 16 * kbl + 8 * hh, 4, 32 * mt + (cc & 16), ln & 15);
            *reinterpret_cast<half8*>(&Pf[(mt * KV_KB + pass * (KV_KB / KV_PASSES) + kbl) * 64 + ln]) = f;
        }
    }
    __syncthreads();   // fragments ready; the flat copy's space becomes the stage buffers

    uint8_t* stage = stage_all + w * 32 * (QUANT ? KV_STAGE_PITCH : KV_OUT_PITCH);
    const float clip = p.clip;

    // one step: 32 tokens whose rows are in `rows`; the rows of the next step are requested into `far`
    auto step = [&](int64_t blk, const u32x4 (&rows)[KV_KB], u32x4 (&far)[KV_KB]) {
        issue(blk + bstep, far);                            // always issued (clamped): exact outstanding-load counts
        __builtin_amdgcn_sched_barrier(0);

        f32x16 acc[KV_MT];
#pragma unroll
        for (int mt = 0; mt < KV_MT; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][r] = 0.0f;
#pragma unroll
        for (int kb = 0; kb < KV_KB; ++kb) {
            const half8 b = __builtin_bit_cast(half8, rows[kb]);
#pragma unroll
            for (int mt = 0; mt < KV_MT; ++mt) {
                const half8 a = *reinterpret_cast<const half8*>(&Pf[(mt * KV_KB + kb) * 64 + l]);
                acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[mt], 0, 0, 0);
            }
        }
        if constexpr (!QUANT) {
            // fp16 rows: a lane holds runs of 8 consecutive channels of its token -> 16-byte LDS writes, then whole
            // 256-byte rows leave with 16-byte stores (lane -> row l/16 + 4k, chunk l%16)
            uint8_t* srow = stage + c * KV_OUT_PITCH;
#pragma unroll
            for (int mt = 0; mt < KV_MT; ++mt)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    half8 v;
#pragma unroll
                    for (int k = 0; k < 8; ++k) v[k] = (_Float16)acc[mt][8 * u + k];
                    *reinterpret_cast<half8*>(srow + 2 * (32 * mt + 16 * u + 8 * h)) = v;
                }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const int64_t g0 = first_group(blk);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int r = (l >> 4) + 4 * k, ch = l & 15;
                const u32x4 v = *reinterpret_cast<const u32x4*>(stage + r * KV_OUT_PITCH + 16 * ch);
                __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p.out_codes + g0 * (2 * KV_D)) + (size_t)group_ofs(blk, r) * (KV_D / 8) + ch);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            return;
        }
        // ---- group range (always containing 0): in-lane over 64 values, then the other half-wave's 64
        float mx = 0.0f, mn = 0.0f;
#pragma unroll
        for (int mt = 0; mt < KV_MT; ++mt)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {   // running value first: each pair folds into one v_max3 / v_min3
                mx = __builtin_fmaxf(__builtin_fmaxf(mx, acc[mt][r]), acc[mt][r + 1]);
                mn = __builtin_fminf(__builtin_fminf(mn, acc[mt][r]), acc[mt][r + 1]);
            }
        mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32));
        mn = __builtin_fminf(mn, __shfl_xor(mn, 32));
        mx *= clip;
        mn *= clip;
        constexpr int QB = BITS ? BITS : 4;                        // (the fp16-out instance never gets here)
        constexpr float LV = (float)((1 << QB) - 1);              // 2^b - 1 intervals
        const _Float16 sh = (_Float16)((mx - mn) * (1.0f / LV));   // round-to-nearest-even to fp16
        const float s = (float)sh;
        const float inv = (s > 0.0f && s <= 65504.0f) ? __builtin_amdgcn_rcpf(s) : 0.0f;
        const float z = __builtin_fminf(__builtin_fmaxf(__builtin_rintf(-mn * inv), 0.0f), LV);
        // q = clamp(round(y / s) + z, 0, LV) = round(clamp(y, -z s, (LV - z) s) / s) + z: clamp, then one fma against
        // 1.5 * 2^23 rounds y / s on its own (ties to even, as the definition has it) and leaves 0x4B400000 + round(y / s)
        // in the register (two's complement in the low bits), so 8 results chain with shift-adds; the constant part
        // (0x4B400000 times the sum of the shifts) comes off and the zero point (z in every field) goes on in one
        // integer addition per 8 codes, all modulo 2^32: every field then holds its code, 0 .. LV, and nothing above.
        const float sl = (inv != 0.0f) ? s : 0.0f;
        const float lim_lo = -z * sl, lim_hi = (LV - z) * sl;
        constexpr float magic = 12582912.0f;
        constexpr uint32_t kMagicBits = 0x4B400000u;
        constexpr uint32_t kFields = 1u + (1u << QB) + (1u << 2 * QB) + (1u << 3 * QB) + (QB == 4 ? 0x11110000u : (1u << 4 * QB) + (1u << 5 * QB) + (1u << 6 * QB) + (1u << 7 * QB));
        const uint32_t chain_fix = (uint32_t)(int)z * kFields - kMagicBits * kFields;

        uint8_t* srow = stage + c * KV_STAGE_PITCH;
#pragma unroll
        for (int mt = 0; mt < KV_MT; ++mt)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                uint32_t bits[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const float yc = __builtin_amdgcn_fmed3f(acc[mt][8 * u + k], lim_lo, lim_hi);
                    bits[k] = __builtin_bit_cast(uint32_t, __builtin_fmaf(yc, inv, magic));
                }
                const uint32_t lo4 = lshl_add(lshl_add(bits[3], QB, bits[2]), 2 * QB, lshl_add(bits[1], QB, bits[0]));
                const uint32_t hi4 = lshl_add(lshl_add(bits[7], QB, bits[6]), 2 * QB, lshl_add(bits[5], QB, bits[4]));
                const uint32_t pk = lshl_add(hi4, 4 * QB, lo4) + chain_fix;   // 8 codes, 8 QB bits
                const int dp = 32 * mt + 16 * u + 8 * h;   // first of 8 consecutive output channels
                if constexpr (QB == 4) {
                    *reinterpret_cast<uint32_t*>(srow + (dp >> 1)) = pk;
                } else if constexpr (QB == 2) {
                    *reinterpret_cast<uint16_t*>(srow + (dp >> 2)) = (uint16_t)pk;
                } else {
                    // 3 bytes at byte 3 dp / 8 = 12 mt + 6 u + 3 h: even for h = 0 (2 bytes, then 1), odd for h = 1 (1, then 2)
                    uint8_t* dst = srow + 12 * mt + 6 * u + 3 * h;
                    *reinterpret_cast<uint16_t*>(dst + h) = (uint16_t)(pk >> (8 * h));
                    dst[2 - 2 * h] = (uint8_t)(pk >> (16 - 16 * h));
                }
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // 32 rows x 16 QB bytes: 16-byte unit q = l + 64k -> (row q / QB, chunk q % QB).  Rows past the end hold a copy of
        // the last token's row (their lanes re-read its input), so they are stored onto it: same bytes, no branch.
        const int64_t g0 = first_group(blk);
        constexpr int NUNIT = 32 * QB;
#pragma unroll
        for (int k = 0; k < (NUNIT + 63) / 64; ++k) {
            const int q = l + 64 * k;
            if (NUNIT % 64 == 0 || q < NUNIT) {
                const int r = q / QB, ch = q % QB;
                const u32x4 v = *reinterpret_cast<const u32x4*>(stage + r * KV_STAGE_PITCH + 16 * ch);
                u32x4* dst = reinterpret_cast<u32x4*>(p.out_codes + g0 * (KV_D * QB / 8)) + (size_t)group_ofs(blk, r) * QB + ch;
                if constexpr (QB == 3) *dst = v;   // 48-byte rows end inside a 32-byte sector: leave them to L2 to merge with their neighbours
                else __builtin_nontemporal_store(v, dst);
            }
        }
        if (h == 0) {   // both half-waves hold the same step and zero point: one of them stores
            const size_t go = group_ofs(blk, c);
            (p.out_scales + g0)[go] = sh;
            (p.out_zeros + g0)[go] = (_Float16)z;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();   // staged rows are consumed before the next step overwrites them
    };
    while (blk < nblk) {
        step(blk, cur, nxt);
        blk += bstep;
        if (blk >= nblk) break;
        step(blk, nxt, cur);
        blk += bstep;
    }
}

template <int BITS>
static hipError_t kv_launch_mode(const KvArgs& a, hipStream_t stream) {
    constexpr int LDS = BITS ? KV_LDS_BYTES : KV_OUT_LDS_BYTES;
    static OccCache occ_cache;
    int occ = 0;
    {
        hipError_t e = kernel_occupancy(reinterpret_cast<const void*>(kv_kernel<BITS>), KV_NT, LDS, occ_cache, occ);
        if (e != hipSuccess) return e;
    }
    // One workgroup per CU (its LDS holds the fragment table and, while that is built, all of P_h).  With P_h staged in
    // two halves two workgroups fit, and measured 5 - 15 % slower from T = 8192 up (twice as many fragment tables to
    // build, four steps per wave instead of eight at 32768 x 8) and the same below.  FLATQUANT_KV_WG_PER_CU caps the
    // number further (0: as many as fit).
    const int cap = env_int("FLATQUANT_KV_WG_PER_CU", 1);
    if (cap > 0 && cap < occ) occ = cap;
    const int64_t nblk = (a.T + KV_TOK - 1) / KV_TOK;
    const int64_t need = (nblk + KV_WAVES - 1) / KV_WAVES;               // workgroups per head if each wave took one step
    int64_t gx = ((int64_t)cu_count() * occ + a.H - 1) / a.H;            // resident workgroups, shared among the heads
    if (gx < 1) gx = 1;
    const int64_t rounds = (need + gx - 1) / gx;                         // same number of steps (+-1) for every workgroup
    gx = (need + rounds - 1) / rounds;
    KvDev d;
    d.kv = a.kv; d.P = a.P; d.out_codes = a.out_codes; d.out_scales = a.out_scales; d.out_zeros = a.out_zeros;
    d.T = a.T; d.H = a.H; d.Hp = a.Hp; d.clip = a.clip;
    return launch(kv_kernel<BITS>, dim3((unsigned)gx, (unsigned)a.H), dim3(KV_NT), LDS, stream, d);
}

hipError_t kv_launch(const KvArgs& a0, hipStream_t stream) {
    // One matrix for all heads (the paper's setting: one P_h per layer): the (token, head) groups are then T * H rows
    // of one head, which a wave takes 32 consecutive ones at a time (8 KB in one piece) instead of 32 rows that lie
    // H * 256 bytes apart.  Same results bit for bit; 32768 x 8 x 128: 23.2 -> 19.9 us.
    KvArgs a = a0;
    if (a.Hp == 1 && a.H > 1 && env_int("FLATQUANT_KV_FOLD_HEADS", 1)) {
        a.T = a.T * a.H;
        a.H = 1;
    }
    if (a.fp16_out) return kv_launch_mode<0>(a, stream);
    switch (a.bits) {
        case 2: return kv_launch_mode<2>(a, stream);
        case 3: return kv_launch_mode<3>(a, stream);
        case 4: return kv_launch_mode<4>(a, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fq
