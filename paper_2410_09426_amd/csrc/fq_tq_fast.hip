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
//   * A wave may own SPW adjacent slabs (template parameter).  With SPW = n2/32 a
//     token belongs to a single wave: no workgroup barrier partner to wait for,
//     and the token tile is read from LDS once instead of once per slab.
#include <type_traits>

#include "fq_internal.h"
#include "fq_device.h"

namespace fq {

__host__ __device__ constexpr int cmax(int a, int b) { return a > b ? a : b; }

// LDS carve-up, shared by host and device.
template <int A, int B, int NBUF = 1, bool MX = false>
struct FastLds {
    static constexpr int N2 = 32 * B;
    static constexpr int PITCH = N2 + kLdsPad;                       // halves per row of the token tile
    static constexpr int XS_BYTES = 32 * A * PITCH * 2;
    // packed codes of one token, one row of X~ (N2 / 2 bytes) per line; 16 bytes of padding per line spread the
    // 2-byte writes of 32 lanes (one line each) over the banks instead of piling them on two
    static constexpr int SPITCH = N2 / 2 + 16;
    static constexpr int STAGE_BYTES = MX ? 32 * A * SPITCH : 0;   // INT4 codes leave from registers
    static constexpr int BODY_BYTES = NBUF * (XS_BYTES + STAGE_BYTES) + 32 * (NBUF < 2 ? 2 : NBUF);   // + one absmax float per wave and buffer
    static constexpr int P2ROWS = (B <= 4) ? N2 : N2 / 2;            // rows of P2 staged per pass
    static constexpr int P2PASSES = N2 / P2ROWS;
    static constexpr int P1FLAT_BYTES = 32 * A * 32 * A * 2;
    static constexpr int STG_BYTES = P1FLAT_BYTES + P2ROWS * N2 * 2;
    static constexpr int R0 = (cmax(BODY_BYTES, STG_BYTES) + 15) & ~15;
    // P1's fragments stay in registers up to three row tiles x six column slabs (86 x 128: 137 -> 130 us at T=16384,
    // 6.7 -> 6.4 us at 64 tokens); beyond that they would spill, and are read from a table in LDS at every use
    static constexpr bool P1LDS = (A >= 4) || (A == 3 && B >= 7);
    static constexpr int P1S_BYTES = P1LDS ? A * 2 * A * 64 * 16 : 0;
    static constexpr int TOTAL = R0 + P1S_BYTES;
};

// KIND 0: persistent loop, one token per step; 1: persistent loop, software-pipelined over tokens;
// 2: one token per workgroup (small T: every token gets its own workgroup, all resident at once, 4 waves per SIMD)
// ID2: the second factor is left out (identity): only the contraction over axis 1 runs, its operand gathered from the
// token tile in LDS with transposing reads (the tile holds exact fp16, so there is no hi / lo split).
// TPW (KIND 2, one wave per token only): tokens per workgroup.  The waves of a workgroup share the staging of P1 and
// P2 (the bytes every workgroup pulls through its CU's vector memory path on top of its tokens) and nothing else:
// after the fragments are built each wave works on its own token, tile and staged codes, with no workgroup barrier.
// MX: MXFP4 output instead of INT4 (the data type the paper's "Limitations" name next; OCP Microscaling format): every
// 32 consecutive channels (one row of X~, one 32-column slab: exactly the 32 values a lane pair (c, 0), (c, 1) holds
// after the second contraction) share a power-of-two scale 2^(floor(log2(alpha max|y|)) - 2), stored as its biased
// exponent; elements are y / scale rounded to E2M1 by v_cvt_scalef32_pk_fp4_f32 (nearest, ties to even, saturating).
// No per-token absmax, so no exchange between waves.  p.out_scales then points at the u8 [T, n/32] exponents.
template <int A, int B, int SPW, bool FULL1, int KIND, bool ID2 = false, int TPW = 1, bool MX = false>
__global__ __launch_bounds__(64 * (B / SPW) * TPW) __attribute__((amdgpu_waves_per_eu((KIND == 2 && SPW == 1) ? 4 : 2))) void tq_fast_kernel(TqDev p, const float* __restrict__ clip) {
    static_assert(B % SPW == 0 && 16 % SPW == 0, "slabs per wave must divide the slab count and 16");
    static_assert(!MX || (KIND != 1 && SPW == 1 && TPW == 1 && !ID2), "MXFP4 output: plain loop or one token per workgroup");
    static_assert(TPW == 1 || (KIND == 2 && B == SPW && A <= 2), "several tokens per workgroup: loop-free kernel, one wave per token");
    constexpr bool PIPE = (KIND == 1), ONE = (KIND == 2);
    using L = FastLds<A, B, PIPE ? 2 : TPW, MX>;
    constexpr int WPT = B / SPW;                  // waves per token
    constexpr int NT = 64 * WPT, NTA = NT * TPW, N2 = L::N2, PITCH = L::PITCH;   // threads per token, per workgroup
    constexpr int KB1 = 2 * A, KB2 = 2 * B, NPRE = 2 * A * SPW;
    constexpr int RSTEP = 16 / SPW;               // rows of X~ covered by one 16-byte chunk per thread
    constexpr int CPR = 4 * B;                    // 16-byte chunks per row of X~
    constexpr bool P1LDS = L::P1LDS;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // body layout: [tile 0][tile 1 if PIPE][stage 0][stage 1 if PIPE][absmax exchange: 8 floats per buffer]
    constexpr int NBUF = PIPE ? 2 : TPW;
    _Float16* Xs = reinterpret_cast<_Float16*>(smem);
    uint8_t* stage = smem + NBUF * L::XS_BYTES;
    float* red = reinterpret_cast<float*>(smem + NBUF * (L::XS_BYTES + L::STAGE_BYTES));
    uint8_t* mxs = smem + L::TOTAL;               // MX only: shared exponents of one token, [32 A rows][B slabs]
    u32x4* P1s = reinterpret_cast<u32x4*>(smem + L::R0);
    _Float16* P1flat = reinterpret_cast<_Float16*>(smem);
    _Float16* P2flat = reinterpret_cast<_Float16*>(smem + L::P1FLAT_BYTES);

    const int tida = threadIdx.x;                 // thread within the workgroup: used where all waves share work
    const int tid = TPW > 1 ? (tida & (NT - 1)) : tida;   // thread within the token's waves
    const int ts = TPW > 1 ? tida / NT : 0;       // token slot of this wave inside the workgroup
    const int l = tid & 63, w = tid >> 6, c = l & 31, h = l >> 5;   // w: wave within the token
    const int n1 = FULL1 ? 32 * A : p.n1;
    const int64_t row_bytes_out = (int64_t)n1 * (N2 / 2);

    // chunk k of this thread: row (tid / CPR) + RSTEP * k of X~, 8 halves at column (tid % CPR) * 8
    const int xrow0 = tid / CPR;
    const int xbase = xrow0 * PITCH + (tid % CPR) * 8;

    auto issue = [&](int64_t t, u32x4 (&pre)[NPRE]) {
        const u32x4* src = reinterpret_cast<const u32x4*>(p.x + t * p.x_stride) + tid;
#pragma unroll
        for (int k = 0; k < NPRE; ++k) {
            int off = k * NT;
            if constexpr (!FULL1) {
                // Rows past n1 (only possible in the last row tile) re-read row n1 - 1: no branch, per lane or per
                // request, so the requests are scheduled as for a full tile.  The products of those tile rows meet
                // all-zero rows of the P1 fragments, so whatever they hold (finite) drops out.
                if (RSTEP * (k + 1) > 32 * (A - 1)) {   // at compile time: last row tile only
                    const int over = xrow0 + RSTEP * k - (n1 - 1);
                    off -= (over > 0 ? over : 0) * CPR;
                }
            }
            pre[k] = __builtin_nontemporal_load(src + off);
        }
    };
    auto commit = [&](const u32x4 (&pre)[NPRE], int buf = 0) {
        _Float16* Xt = Xs + buf * (L::XS_BYTES / 2);
#pragma unroll
        for (int k = 0; k < NPRE; ++k) {
            *reinterpret_cast<u32x4*>(Xt + xbase + RSTEP * k * PITCH) = pre[k];
        }
    };

    // ---- the first token row of this workgroup is requested before anything else
    constexpr bool DEEP = !ONE && (PIPE || (NPRE <= 4));   // two rows in flight per workgroup when the registers allow it
    u32x4 pre0[NPRE], pre1[DEEP ? NPRE : 1];
    int64_t t = (int64_t)blockIdx.x * TPW + ts;
    const int64_t G = gridDim.x;
    const bool live = TPW == 1 || t < p.T;        // a last workgroup's spare waves redo token T - 1 and store nothing
    if (TPW > 1 && !live) t = p.T - 1;
    issue(t, pre0);

    // ---- stage P1 (flat, n1 x n1) and P2 (in one or two passes of rows) in LDS with coalesced loads.  All loads of
    // a stage are issued before any of them is consumed, so the stage costs one memory latency, not one per element.
    // `after_first_loads()` runs once, right after the first batch of loads has been issued and before anything waits
    // for it: the place to queue further requests that nothing in the prologue depends on.
    auto stage_p1 = [&](auto&& after_first_loads) {
        const int n1sq = n1 * n1;
        bool queued = false;               // after_first_loads() has run
        // `count` units from `src`, a batch of 8 per thread in flight; store(idx, unit) puts one into LDS
        auto copy_batched = [&](auto batch, const auto* src, int count, auto&& store) {
            constexpr int BATCH = decltype(batch)::value;
            using Unit = decltype(*src + 0);
            for (int base = 0; base < count; base += BATCH * NTA) {
                Unit v[BATCH];
#pragma unroll
                for (int k = 0; k < BATCH; ++k) {
                    const int idx = base + k * NTA + tida;
                    v[k] = src[idx < count ? idx : count - 1];
                }
                if (base == 0) {
                    __builtin_amdgcn_sched_barrier(0);
                    after_first_loads();
                    queued = true;
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int k = 0; k < BATCH; ++k) {
                    const int idx = base + k * NTA + tida;
                    if (idx < count) store(idx, v[k]);
                }
            }
        };
        if constexpr (FULL1) {   // the LDS copy is the matrix as it is
            if ((reinterpret_cast<uintptr_t>(p.P1) & 15) == 0) {
                copy_batched(std::integral_constant<int, 8>{}, reinterpret_cast<const u32x4*>(p.P1), n1sq >> 3, [&](int idx, u32x4 v) { reinterpret_cast<u32x4*>(P1flat)[idx] = v; });
            } else {             // only 4-byte aligned: pairs
                copy_batched(std::integral_constant<int, 8>{}, reinterpret_cast<const uint32_t*>(p.P1), n1sq >> 1, [&](int idx, uint32_t v) { reinterpret_cast<uint32_t*>(P1flat)[idx] = v; });
            }
        } else {
            // Rows re-pitched to PW = n1 rounded up to whole row tiles, the padding zero.  One short code path (these
            // launches are latency-bound and every instruction line is fetched cold; a variant that moves 16-byte
            // chunks and places their four pairs was slower): pairs of elements, P1 being 4-byte aligned, 16 of them per
            // thread in flight (one batch up to n1 = 90), each half written on its own since a pair straddles two rows
            // when n1 is odd; floor(f / n1) = umulhi(f, magic) for f < 2^16, the magic number comes from the host.
            constexpr int PW = 32 * A;
            uint16_t* dst = reinterpret_cast<uint16_t*>(P1flat);
            for (int q = tida; q < (PW - n1) * PW / 8; q += NTA) reinterpret_cast<u32x4*>(P1flat + n1 * PW)[q] = u32x4{0u, 0u, 0u, 0u};
            for (int r = tida; r < n1; r += NTA)
                for (int cc = n1; cc < PW; ++cc) dst[r * PW + cc] = 0;
            const uint32_t magic = p.n1_magic;
            const uint16_t tail = reinterpret_cast<const uint16_t*>(p.P1)[n1sq - 1];
            copy_batched(std::integral_constant<int, 16>{}, reinterpret_cast<const uint32_t*>(p.P1), n1sq >> 1, [&](int idx, uint32_t v) {
                const uint32_t f = 2u * (uint32_t)idx;
                const int row = (int)__umulhi(f, magic), col = (int)f - row * n1, a0 = row * PW + col;
                dst[a0] = (uint16_t)v;
                dst[a0 + 1 + (col + 1 == n1 ? PW - n1 : 0)] = (uint16_t)(v >> 16);
            });
            if ((n1sq & 1) && tida == 0) dst[(n1 - 1) * PW + n1 - 1] = tail;
        }
        if (!queued) after_first_loads();   // a P1 of fewer elements than one load unit (n1 = 1): no batch ran
    };
    half8 p2f[ID2 ? 1 : SPW][ID2 ? 1 : KB2];
    half8 p1f[P1LDS ? 1 : A][P1LDS ? 1 : KB1];
#pragma unroll
    for (int pass = 0; pass < (ID2 ? 1 : L::P2PASSES); ++pass) {
        constexpr int CH = L::P2ROWS * N2 / 8;
        const u32x4* src = reinterpret_cast<const u32x4*>(p.P2) + pass * CH;
        static_assert(CH % NTA == 0, "P2 pass divides over the workgroup's threads");
        u32x4 v2[CH / NTA];
        if constexpr (!ID2) {
#pragma unroll
            for (int k = 0; k < CH / NTA; ++k) v2[k] = src[tida + k * NTA];
        }
        if (pass == 0) {
            // P1's loads queue behind P2's: one latency for both.  The second token row is requested behind them, so
            // it is in flight during the whole prologue without delaying the transforms (loads return in order).
            stage_p1([&]() {
                if constexpr (PIPE) issue((t + G < p.T) ? t + G : p.T - 1, pre1);
                else if constexpr (DEEP) { if (t + G < p.T) issue(t + G, pre1); }
            });
        }
        else __syncthreads();               // previous pass fully consumed
        if constexpr (!ID2) {
#pragma unroll
            for (int k = 0; k < CH / NTA; ++k) reinterpret_cast<u32x4*>(P2flat)[tida + k * NTA] = v2[k];
        }
        __syncthreads();
        // B-operand fragments of this wave's slab: lane (c, h) holds P2[16kb + 8h + s][32w + c], s = 0..7
        if constexpr (!ID2) {
#pragma unroll
            for (int kb = pass * (L::P2ROWS / 16); kb < (pass + 1) * (L::P2ROWS / 16); ++kb)
#pragma unroll
                for (int q = 0; q < SPW; ++q)
                    p2f[q][kb] = lds_column8(P2flat, N2, 16 * kb - pass * L::P2ROWS + 8 * h, 4, 32 * (w * SPW + q) + (c & 16), l & 15);
        }
        if (pass == 0) {
            // P1 fragments, gathered with the k-permutation of the first contraction's accumulator layout:
            // K block kk, slot s, half-wave h  <->  i = 32(kk/2) + 8(2(kk%2) + s/4) + 4h + s%4.  The LDS copy is padded with
            // zeros to whole row tiles, so ragged factors take the same transposing reads as full ones.
            if constexpr (P1LDS) {
                for (int e = tid; e < A * KB1 * 64; e += NT) {   // e % 64 is the lane: whole 16-lane blocks cooperate in the reads
                    const int ln = e & 63, kk = (e >> 6) % KB1, It = (e >> 6) / KB1;
                    const int cc = ln & 31, hh = ln >> 5;
                    const half8 f = lds_column8(P1flat, 32 * A, 32 * (kk >> 1) + 16 * (kk & 1) + 4 * hh, 8, 32 * It + (cc & 16), ln & 15);
                    *reinterpret_cast<half8*>(&P1s[e]) = f;
                }
            } else {
#pragma unroll
                for (int It = 0; It < A; ++It)
#pragma unroll
                    for (int kk = 0; kk < KB1; ++kk)
                        p1f[It][kk] = lds_column8(P1flat, 32 * A, 32 * (kk >> 1) + 16 * (kk & 1) + 4 * h, 8, 32 * It + (c & 16), l & 15);
            }
        }
    }
    __syncthreads();   // staging area is free: it becomes the token tile
    // with one wave per token the tile, the staged codes and the absmax slot of a token are touched by that wave only:
    // LDS executes a wave's instructions in order, so program order is all that has to be kept
    auto token_sync = [&]() {
        if constexpr (TPW > 1) {
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        } else {
            __syncthreads();
        }
    };
    commit(pre0, ts);
    token_sync();

    // ---- both contractions for the token tile in LDS buffer `buf`: acc2 = (P1^T X~ P2)^T for this wave's slabs
    // `side(slot)` is called NSLOT times at even intervals of the MFMA stream; the pipelined loop uses it to
    // interleave the previous token's rounding and packing (vector ALU only) with this token's MFMAs.
    constexpr int NSLOT1 = SPW * ((A + 1) / 2) * KB2, NSLOT = NSLOT1 + SPW * A * 2;
    auto gemm = [&](int buf, f32x16 (&acc2)[SPW][A], auto&& side) {
        const _Float16* Xt = Xs + buf * (L::XS_BYTES / 2);
#pragma unroll
        for (int q = 0; q < SPW; ++q)
#pragma unroll
            for (int It = 0; It < A; ++It)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc2[q][It][r] = 0.0f;
        if constexpr (ID2) {
            // Z = X~: lane (c, h) takes, for K block kk, the 8 tile rows of the accumulator-layout permutation in its
            // own column, i.e. the same gather as for the P1 fragments, straight from the token tile
            static_assert(!P1LDS, "left-factor-only variant keeps the P1 fragments in registers");
#pragma unroll
            for (int q = 0; q < SPW; ++q)
#pragma unroll
                for (int kk = 0; kk < KB1; ++kk)
                    if (FULL1 || 16 * kk < n1) {
                        const half8 z = lds_column8(Xt, PITCH, 32 * (kk >> 1) + 16 * (kk & 1) + 4 * h, 8, 32 * (w * SPW + q) + (c & 16), l & 15);
#pragma unroll
                        for (int It = 0; It < A; ++It) acc2[q][It] = __builtin_amdgcn_mfma_f32_32x32x16_f16(z, p1f[It][kk], acc2[q][It], 0, 0, 0);
                    }
#pragma unroll
            for (int slot = 0; slot < NSLOT; ++slot) side(slot);
            return;
        }
        // row tiles of X~ go through the first contraction in pairs so that consecutive MFMAs are independent
#pragma unroll
        for (int q = 0; q < SPW; ++q)
#pragma unroll
        for (int I0 = 0; I0 < A; I0 += 2) {
            constexpr int NI_MAX = 2;
            const int ni = (A - I0) < NI_MAX ? (A - I0) : NI_MAX;
            f32x16 acc1[NI_MAX];
#pragma unroll
            for (int d = 0; d < NI_MAX; ++d)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc1[d][r] = 0.0f;
            const _Float16* arow = Xt + (32 * I0 + c) * PITCH + 8 * h;
            if constexpr (A >= 3) {
                // wide tiles: the operands of K block kb + 1 are read from LDS before the MFMAs of block kb are issued
                // (measured: helps the 128-row tiles, costs the 64-row ones)
                half8 anext[NI_MAX];
#pragma unroll
                for (int d = 0; d < NI_MAX; ++d)
                    if (d < ni) anext[d] = *reinterpret_cast<const half8*>(arow + d * 32 * PITCH);
#pragma unroll
                for (int kb = 0; kb < KB2; ++kb) {
                    half8 acur[NI_MAX];
#pragma unroll
                    for (int d = 0; d < NI_MAX; ++d)
                        if (d < ni) acur[d] = anext[d];
                    if (kb + 1 < KB2) {
#pragma unroll
                        for (int d = 0; d < NI_MAX; ++d)
                            if (d < ni) anext[d] = *reinterpret_cast<const half8*>(arow + d * 32 * PITCH + 16 * (kb + 1));
                        __builtin_amdgcn_sched_barrier(0);
                    }
#pragma unroll
                    for (int d = 0; d < NI_MAX; ++d)
                        if (d < ni) acc1[d] = __builtin_amdgcn_mfma_f32_32x32x16_f16(acur[d], p2f[q][kb], acc1[d], 0, 0, 0);
                    side((q * ((A + 1) / 2) + I0 / 2) * KB2 + kb);
                }
            } else {
#pragma unroll
                for (int kb = 0; kb < KB2; ++kb) {
#pragma unroll
                    for (int d = 0; d < NI_MAX; ++d)
                        if (d < ni) {
                            const half8 a = *reinterpret_cast<const half8*>(arow + d * 32 * PITCH + 16 * kb);
                            acc1[d] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, p2f[q][kb], acc1[d], 0, 0, 0);
                        }
                    side((q * ((A + 1) / 2) + I0 / 2) * KB2 + kb);
                }
            }
            // Y^T[slab, :] += Z^T[slab, K block] P1[K block, :], hi and lo parts of Z
#pragma unroll
            for (int d = 0; d < NI_MAX; ++d)
#pragma unroll
                for (int kq = 0; kq < 2; ++kq) {
                    const int kk = 2 * (I0 + d) + kq;
                    // K blocks past n1 meet all-zero rows of the P1 fragments: multiplied like the others, except with four
                    // row tiles, where the kernel is MFMA-bound and a skipped block (112 rows: one of eight) pays for its branch
                    if (d < ni && (FULL1 || A < 4 || 16 * kk < n1)) {
                        half8 zh, zl;
                        split_hi_lo(acc1[d], 8 * kq, zh, zl);
                        half8 b[A];
#pragma unroll
                        for (int It = 0; It < A; ++It) {
                            if constexpr (P1LDS) b[It] = *reinterpret_cast<const half8*>(&P1s[(It * KB1 + kk) * 64 + l]);
                            else b[It] = p1f[It][kk];
                        }
#pragma unroll
                        for (int It = 0; It < A; ++It) acc2[q][It] = __builtin_amdgcn_mfma_f32_32x32x16_f16(zh, b[It], acc2[q][It], 0, 0, 0);
#pragma unroll
                        for (int It = 0; It < A; ++It) acc2[q][It] = __builtin_amdgcn_mfma_f32_32x32x16_f16(zl, b[It], acc2[q][It], 0, 0, 0);
                    }
                    if (d < ni) side(NSLOT1 + (q * A + I0 + d) * 2 + kq);
                }
        }
    };

    // ---- this wave's share of the per-token absmax (in-lane, then DPP over the wave), left in red[buf][w]
    auto absmax_to_lds = [&](const f32x16 (&acc2)[SPW][A], int buf) {
        float m = 0.0f;
#pragma unroll
        for (int q = 0; q < SPW; ++q)
#pragma unroll
            for (int It = 0; It < A; ++It)
#pragma unroll
                for (int r = 0; r < 16; ++r) m = __builtin_fmaxf(m, __builtin_fabsf(acc2[q][It][r]));
        m = wave_max(m);
        if (l == 0) red[buf * 8 + w] = m;
    };
    auto absmax_from_lds = [&](int buf) {
        float m = 0.0f;
#pragma unroll
        for (int b = 0; b < WPT; ++b) m = __builtin_fmaxf(m, red[buf * 8 + b]);
        return m;
    };

    // ---- step from the absmax; round, clamp, pack, store.  INT4 codes leave from registers.  v_cvt_pknorm_i16_f32
    // (clamp to [-1, 1], times 32767, round to nearest) applied to r = (4096 (u + 0.5) - 0.5) / 32767, u = y / step,
    // leaves clamp(rne(u), -8, 7) as the two's-complement top nibble of a 16-bit field: clamping, rounding and half of
    // the packing cost one fma plus half an instruction per value.  (The thresholds between codes move by less than
    // 2e-6 code units: fp32 rounding of the two constants and of the fma.)
    const int stage_lane = c * L::SPITCH + ((32 * w * SPW + 4 * h) >> 1);   // MXFP4 path: this lane's byte offset inside the staged codes
    struct Step { _Float16 sh; float kmul; };
    auto make_step = [&](float m, float clipv) {
        Step st;
        st.sh = (_Float16)(clipv * m * 0.142857149f);   // step = alpha * max / 7, round-to-nearest-even to fp16
        const float s = (float)st.sh;
        const float inv = (s > 0.0f && s <= 65504.0f) ? __builtin_amdgcn_rcpf(s) : 0.0f;   // 1 ulp: < 1e-6 code units
        st.kmul = inv * (4096.0f / 32767.0f);
        return st;
    };
    // One unit = 8 channels of one lane (accumulator registers 8 mm .. 8 mm + 7 of slab q, row tile It: channels
    // 32 (w SPW + q) + 8 g + 4 h + k, g = 2 mm, 2 mm + 1) -> one dword of nibbles.  When a row tile's units are done, one
    // exchange between the half-waves (v_permlane32_swap) turns the lane pair's alternating 2-byte pieces into 8 (one
    // slab per wave) or 16 (two slabs) consecutive bytes of the code row per lane, which are stored at once.
    constexpr int NUNIT = SPW * A * 2;
    constexpr float kadd = 2047.5f / 32767.0f;
    uint32_t Wq[SPW][A][2];
    auto quant_unit = [&](const f32x16 (&acc2)[SPW][A], const Step& st, int64_t tok, int u) {
        const int q = u / (2 * A), It = (u / 2) % A, mm = u % 2;
        uint32_t D[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float r0 = __builtin_fmaf(acc2[q][It][8 * mm + k], st.kmul, kadd);
            const float r1 = __builtin_fmaf(acc2[q][It][8 * mm + 4 + k], st.kmul, kadd);
            D[k] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pknorm_i16(r0, r1));
        }
        // bytes 1 and 3 of D[k] carry nibbles k and k + 4 on top: even nibbles -> E, odd ones -> F
        const uint32_t E = __builtin_amdgcn_perm(D[2], D[0], 0x07030501u);
        const uint32_t F = __builtin_amdgcn_perm(D[3], D[1], 0x07030501u);
        Wq[q][It][mm] = (F & 0xF0F0F0F0u) | ((E >> 4) & 0x0F0F0F0Fu);
        if (mm == 1 && q == SPW - 1) {
            const int ip = 32 * It + c;
            uint8_t* dst = p.out_codes + tok * row_bytes_out + ip * (N2 / 2) + 16 * (w * SPW + (SPW == 2 ? h : 0)) + (SPW == 1 ? 8 * h : 0);
            if constexpr (SPW == 1) {
                // afterwards half-wave 0 holds the groups g = 0, 1 of both lanes of the pair, half-wave 1 the groups 2, 3
                const auto sw = __builtin_amdgcn_permlane32_swap(Wq[0][It][0], Wq[0][It][1], false, false);
                uint2 o;
                o.x = __builtin_amdgcn_perm(sw[1], sw[0], 0x05040100u);
                o.y = __builtin_amdgcn_perm(sw[1], sw[0], 0x07060302u);
                if (FULL1 || ip < n1) *reinterpret_cast<uint2*>(dst) = o;
            } else {
                // afterwards half-wave h holds slab q = h of both lanes of the pair
                u32x4 o;
#pragma unroll
                for (int m2 = 0; m2 < 2; ++m2) {
                    const auto sw = __builtin_amdgcn_permlane32_swap(Wq[0][It][m2], Wq[1][It][m2], false, false);
                    o[2 * m2] = __builtin_amdgcn_perm(sw[1], sw[0], 0x05040100u);
                    o[2 * m2 + 1] = __builtin_amdgcn_perm(sw[1], sw[0], 0x07060302u);
                }
                if (FULL1 || ip < n1) *reinterpret_cast<u32x4*>(dst) = o;
            }
        }
    };
    // all of a token's codes, then its step (every lane writes the same two bytes: cheaper than a branch around the store)
    auto quant_store = [&](const f32x16 (&acc2)[SPW][A], float m, float clipv, int64_t tok) {
        const Step st = make_step(m, clipv);
#pragma unroll
        for (int u = 0; u < NUNIT; ++u) quant_unit(acc2, st, tok, u);
        p.out_scales[tok] = st.sh;
    };
    // MXFP4: per (row of X~, slab) block of 32 channels; 4 consecutive channels of a lane -> 2 bytes, as for INT4
    auto mx_quant_to_stage = [&](const f32x16 (&acc2)[SPW][A], float clipv) {
        uint8_t* stg = stage;
#pragma unroll
        for (int q = 0; q < SPW; ++q)
#pragma unroll
            for (int It = 0; It < A; ++It) {
                float m = 0.0f;
#pragma unroll
                for (int r = 0; r < 16; r += 2) m = __builtin_fmaxf(__builtin_fmaxf(m, __builtin_fabsf(acc2[q][It][r])), __builtin_fabsf(acc2[q][It][r + 1]));
                m = __builtin_fmaxf(m, __shfl_xor(m, 32)) * clipv;
                const int be = (int)((__builtin_bit_cast(uint32_t, m) >> 23) & 0xffu);   // biased exponent of alpha * max
                const int e = be > 2 ? be - 2 : 0;
                // the conversion reads the exponent field of its scale operand only, and field 0 means 2^-127 (measured),
                // so the stored exponent is also the one the elements are converted with, down to the bottom of the range
                const float scale = __builtin_bit_cast(float, (uint32_t)e << 23);
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    uint32_t pk = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(0u, acc2[q][It][4 * g], acc2[q][It][4 * g + 1], scale, 0);
                    pk = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(pk, acc2[q][It][4 * g + 2], acc2[q][It][4 * g + 3], scale, 1);
                    *reinterpret_cast<uint16_t*>(stg + stage_lane + 32 * It * L::SPITCH + (32 * q + 8 * g) / 2) = (uint16_t)pk;
                }
                if (h == 0) mxs[(32 * It + c) * B + w * SPW + q] = (uint8_t)e;
            }
    };
    // ---- MXFP4 path: staged codes of token t -> global memory with 16-byte stores; no branch around the stores when
    // the row divides evenly, so that the compiler's count of outstanding memory operations stays exact
    auto copy_out = [&](int64_t t, int buf, _Float16 sh) {
        const u32x4* stg = reinterpret_cast<const u32x4*>(stage + buf * L::STAGE_BYTES);
        u32x4* dst = reinterpret_cast<u32x4*>(p.out_codes + t * row_bytes_out);
        constexpr int NQ_FULL = 32 * A * B;   // 16-byte units of one code row when n1 = 32A
        if constexpr (FULL1 && NQ_FULL % NT == 0) {
#pragma unroll
            for (int k = 0; k < NQ_FULL / NT; ++k) {
                const int q = tid + k * NT;            // unit q = 16-byte chunk q % B of line q / B
                __builtin_nontemporal_store(stg[(q / B) * (B + 1) + q % B], dst + q);
            }
        } else {
            const int nq = n1 * B;
            for (int q = tid; q < nq; q += NT) __builtin_nontemporal_store(stg[(q / B) * (B + 1) + q % B], dst + q);
        }
        if constexpr (MX) {   // n1 * B exponent bytes of the token, a multiple of 4 (checked on the host)
            if (p.mx_tiled) {
                // tile order of the MXFP4 product: rows in tiles of 128; per tile and K iteration (256 channels = 8
                // exponents) the 128 rows' 8 bytes are contiguous: byte (((t / 128) KI + j) 128 + t % 128) 8 + b
                const uint2* src = reinterpret_cast<const uint2*>(mxs);
                const int ki = n1 * B / 8;   // a whole number of iterations (checked on the host)
                uint2* dsc = reinterpret_cast<uint2*>(p.out_scales) + (t >> 7) * ((int64_t)ki * 128) + (t & 127);
                for (int j = tid; j < ki; j += NT) dsc[(int64_t)j * 128] = src[j];
            } else {
                const uint32_t* src = reinterpret_cast<const uint32_t*>(mxs);
                uint32_t* dsc = reinterpret_cast<uint32_t*>(reinterpret_cast<uint8_t*>(p.out_scales) + t * ((int64_t)n1 * B));
                for (int i = tid; i < n1 * B / 4; i += NT) dsc[i] = src[i];
            }
        } else {
            p.out_scales[t] = sh;   // every lane writes the same two bytes: cheaper than a branch around the store
        }
    };
    // Requests are always issued (past the end they re-read the last row): an unconditional request lets the
    // compiler count outstanding loads exactly, so a later wait covers only the older row.
    auto issue_clamped = [&](int64_t tf, u32x4 (&pre)[NPRE]) {
        issue(tf < p.T ? tf : p.T - 1, pre);
        __builtin_amdgcn_sched_barrier(0);   // keep the requests here, ahead of the MFMA work, with their registers reserved
    };

    if constexpr (ONE) {
        const float clipv = clip[p.clip_mode ? t : 0];
        f32x16 acc2[SPW][A];
        gemm(ts, acc2, [](int) {});
        if constexpr (MX) {
            mx_quant_to_stage(acc2, clipv);
            token_sync();
            if (live) copy_out(t, ts, (_Float16)0.0f);
        } else {
            absmax_to_lds(acc2, ts);
            token_sync();
            const float m = absmax_from_lds(ts);
            if (live) quant_store(acc2, m, clipv, t);
        }
    } else if constexpr (!PIPE) {
        // One token per step: the tile of token t is in LDS, `pre_next` holds (or is receiving) the row of token t + G
        // and is written to LDS once every wave is done with the current tile; the row of token t + 2G is requested
        // into `pre_far`.  The caller alternates the two register sets.
        auto body = [&](int64_t t, u32x4 (&pre_next)[NPRE], u32x4 (&pre_far)[NPRE]) {
            issue_clamped(t + (DEEP ? 2 : 1) * G, pre_far);
            const float clipv = clip[p.clip_mode ? t : 0];   // wave-uniform address, read-only: a scalar load
            f32x16 acc2[SPW][A];
            gemm(0, acc2, [](int) {});
            if constexpr (!MX) absmax_to_lds(acc2, 0);
            __syncthreads();   // (A) every wave is also done reading the token tile
            if constexpr (MX) {
                mx_quant_to_stage(acc2, clipv);
                commit(pre_next);   // past the end this is the re-read last row; nobody uses it
                __syncthreads();    // (B) staged codes and the next tile are visible
                copy_out(t, 0, (_Float16)0.0f);
            } else {
                const float m = absmax_from_lds(0);
                quant_store(acc2, m, clipv, t);
                commit(pre_next);
                __syncthreads();    // (B) the next tile is visible
            }
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
    } else {
        // Software-pipelined over tokens: while the MFMA pipe works on token j+1, the vector ALU rounds and packs
        // token j, and there is a single workgroup barrier per token.  Token j's tile, staged codes and absmax
        // slots live in LDS buffer j % 2.  Register sets: pre0 receives tokens t0, t2, ..., pre1 receives t1, t3, ...
        f32x16 accX[SPW][A], accY[SPW][A];
        // prime: token t0 through the contractions; t1's row into tile 1; t2's row requested
        issue_clamped(t + 2 * G, pre0);
        gemm(0, accX, [](int) {});
        absmax_to_lds(accX, 0);
        commit(pre1, 1);
        __syncthreads();
        float m_cur = absmax_from_lds(0);
        float clip_cur = clip[p.clip_mode ? t : 0];
        // step j (token t = t_j in acc_cur): request t_{j+3}; contractions for t_{j+1} overlap with quantizing t_j;
        // t_{j+2}'s row, which arrived during the previous step, replaces t_j's tile
        auto step = [&](int64_t t, int jb, f32x16 (&acc_cur)[SPW][A], f32x16 (&acc_next)[SPW][A],
                        u32x4 (&pre_commit)[NPRE], u32x4 (&pre_issue)[NPRE]) {
            issue_clamped(t + 3 * G, pre_issue);
            const int64_t tn = (t + G < p.T) ? t + G : p.T - 1;
            const float clip_next = clip[p.clip_mode ? tn : 0];
            const Step st = make_step(m_cur, clip_cur);
            gemm(jb ^ 1, acc_next, [&](int slot) {
#pragma unroll
                for (int u = slot * NUNIT / NSLOT; u < (slot + 1) * NUNIT / NSLOT; ++u) quant_unit(acc_cur, st, t, u);
            });
            absmax_to_lds(acc_next, jb ^ 1);
            commit(pre_commit, jb);
            __syncthreads();          // the next tile and the absmax partials are visible
            p.out_scales[t] = st.sh;
            m_cur = absmax_from_lds(jb ^ 1);
            clip_cur = clip_next;
        };
        while (true) {
            if (t + G >= p.T) { quant_store(accX, m_cur, clip_cur, t); break; }
            step(t, 0, accX, accY, pre0, pre1);
            t += G;
            if (t + G >= p.T) { quant_store(accY, m_cur, clip_cur, t); break; }
            step(t, 1, accY, accX, pre1, pre0);
            t += G;
        }
    }
}

// ------------------------------------------------------------------------------------
using KernelFn = void (*)(TqDev, const float*);

struct Variant {
    KernelFn fn;
    int lds;
};

// mode 0: one slab per wave; mode 1: two slabs per wave; mode 2: one slab per wave, software-pipelined over tokens;
// mode 3: one slab per wave, one token per workgroup (only when every token can have a resident workgroup);
// mode 4 (n2 = 64): one wave per token, kTokensPerWg tokens per workgroup sharing the staged transforms, no loop
constexpr int kTokensPerWg = 4;
template <int A, int B>
static Variant variant_ab(bool full1, int mode) {
    if constexpr (A <= 2 && (B == 2 || B == 4 || B == 8)) {
        if (mode == 1)
            return full1 ? Variant{&tq_fast_kernel<A, B, 2, true, 0>, FastLds<A, B>::TOTAL}
                         : Variant{&tq_fast_kernel<A, B, 2, false, 0>, FastLds<A, B>::TOTAL};
    }
    if constexpr (A <= 2 && B == 2) {
        if (mode == 4)
            return full1 ? Variant{&tq_fast_kernel<A, B, 2, true, 2, false, kTokensPerWg>, FastLds<A, B, kTokensPerWg>::TOTAL}
                         : Variant{&tq_fast_kernel<A, B, 2, false, 2, false, kTokensPerWg>, FastLds<A, B, kTokensPerWg>::TOTAL};
    }
    if constexpr (A <= 2) {
        if (mode == 2)
            return full1 ? Variant{&tq_fast_kernel<A, B, 1, true, 1>, FastLds<A, B, 2>::TOTAL}
                         : Variant{&tq_fast_kernel<A, B, 1, false, 1>, FastLds<A, B, 2>::TOTAL};
        if (mode == 3)
            return full1 ? Variant{&tq_fast_kernel<A, B, 1, true, 2>, FastLds<A, B>::TOTAL}
                         : Variant{&tq_fast_kernel<A, B, 1, false, 2>, FastLds<A, B>::TOTAL};
    }
    return full1 ? Variant{&tq_fast_kernel<A, B, 1, true, 0>, FastLds<A, B>::TOTAL}
                 : Variant{&tq_fast_kernel<A, B, 1, false, 0>, FastLds<A, B>::TOTAL};
}

template <int A>
static Variant variant_a(int B, bool full1, int mode) {
    switch (B) {
        case 1: return variant_ab<A, 1>(full1, mode);
        case 2: return variant_ab<A, 2>(full1, mode);
        case 3: return variant_ab<A, 3>(full1, mode);
        case 4: return variant_ab<A, 4>(full1, mode);
        case 5: return variant_ab<A, 5>(full1, mode);
        case 6: return variant_ab<A, 6>(full1, mode);
        case 7: return variant_ab<A, 7>(full1, mode);
        default: return variant_ab<A, 8>(full1, mode);
    }
}

static Variant variant(int A, int B, bool full1, int mode) {
    switch (A) {
        case 1: return variant_a<1>(B, full1, mode);
        case 2: return variant_a<2>(B, full1, mode);
        case 3: return variant_a<3>(B, full1, mode);
        default: return variant_a<4>(B, full1, mode);
    }
}

// MXFP4 output: n2 a multiple of 32; loop-free kernel while every token gets a resident workgroup (64-wide rows), else
// the plain persistent loop.  The shared exponents of a token are staged in LDS behind the kernel's usual carve-up.
template <int A, int B>
static Variant variant_mx_ab(bool full1, bool one) {
    if constexpr (A <= 2 && B == 2) {
        if (one && full1) return Variant{&tq_fast_kernel<A, B, 1, true, 2, false, 1, true>, FastLds<A, B, 1, true>::TOTAL + 32 * A * B};
    }
    return full1 ? Variant{&tq_fast_kernel<A, B, 1, true, 0, false, 1, true>, FastLds<A, B, 1, true>::TOTAL + 32 * A * B}
                 : Variant{&tq_fast_kernel<A, B, 1, false, 0, false, 1, true>, FastLds<A, B, 1, true>::TOTAL + 32 * A * B};
}

template <int A>
static Variant variant_mx_a(int B, bool full1, bool one) {
    switch (B) {
        case 1: return variant_mx_ab<A, 1>(full1, one);
        case 2: return variant_mx_ab<A, 2>(full1, one);
        case 3: return variant_mx_ab<A, 3>(full1, one);
        case 4: return variant_mx_ab<A, 4>(full1, one);
        case 5: return variant_mx_ab<A, 5>(full1, one);
        case 6: return variant_mx_ab<A, 6>(full1, one);
        case 7: return variant_mx_ab<A, 7>(full1, one);
        default: return variant_mx_ab<A, 8>(full1, one);
    }
}

static Variant variant_mx(int A, int B, bool full1, bool one) {
    switch (A) {
        case 1: return variant_mx_a<1>(B, full1, one);
        case 2: return variant_mx_a<2>(B, full1, one);
        case 3: return variant_mx_a<3>(B, full1, one);
        default: return variant_mx_a<4>(B, full1, one);
    }
}

bool tq_mx_applicable(const TqDev& d) {
    if (d.n2 % 32 != 0 || d.n2 < 32 || d.n2 > kMaxN2 || d.n1 < 1 || d.n1 > kMaxN1) return false;
    if (((int64_t)d.n1 * d.n2) % 128 != 0 || !d.vec8 || !d.out_vec16 || !d.P1 || !d.P2) return false;
    if ((reinterpret_cast<uintptr_t>(d.P2) & 15) || (reinterpret_cast<uintptr_t>(d.P1) & 3)) return false;
    return (reinterpret_cast<uintptr_t>(d.out_scales) & 3) == 0;
}

hipError_t tq_mx_launch(const TqDev& d, hipStream_t stream) {
    {   // 64-wide rows: the wave-per-token kernel with the MXFP4 quantizer (modes as for INT4; the tile order of the
        // exponents needs whole K iterations of 256 channels, which 32 x 64 and 64 x 64 have)
        const int m = env_int("FLATQUANT_MODE", -1);
        if ((m == -1 || m == 5 || m == 6) && tq_wave_applicable(d) && (reinterpret_cast<uintptr_t>(d.out_scales) & 7) == 0)
            return tq_wave_launch(d, stream, env_int("FLATQUANT_WAVE_TPW", 4), m == -1 ? d.T >= 32768 : m == 6, true);
    }
    const int A = (d.n1 + 31) / 32, B = d.n2 / 32;
    const bool full1 = (d.n1 % 32) == 0;
    static OccCache occ_cache[4][8][2][2];
    auto occupancy = [&](bool one, int& occ) -> hipError_t {
        const Variant v = variant_mx(A, B, full1, one);
        return kernel_occupancy(reinterpret_cast<const void*>(v.fn), 64 * B, v.lds, occ_cache[A - 1][B - 1][full1][one], occ);
    };
    bool one = false;
    int occ = 0;
    if (A <= 2 && B == 2 && full1 && d.T <= 0x7fffffff) {
        hipError_t e = occupancy(true, occ);
        if (e != hipSuccess) return e;
        one = d.T <= (int64_t)cu_count() * occ;
        const int force = env_int("FLATQUANT_MODE", -1);
        if (force == 0) one = false;
        if (force == 3) one = true;
    }
    if (!one) {
        hipError_t e = occupancy(false, occ);
        if (e != hipSuccess) return e;
    }
    const Variant v = variant_mx(A, B, full1, one);
    int64_t grid = d.T;
    if (!one) {
        const int64_t resident = (int64_t)cu_count() * occ;
        const int64_t rounds = (d.T + resident - 1) / resident;
        grid = (d.T + rounds - 1) / rounds;
    }
    return launch(v.fn, dim3((unsigned)grid), dim3(64 * B), v.lds, stream, d, d.clip);
}

bool tq_fast_applicable(const TqDev& d) {
    if (d.n2 % 32 != 0 || !d.vec8 || !d.out_vec16) return false;
    // a left-out factor (identity): only the left-factor-only case of 128-wide rows (P_o: heads x head_dim) has
    // specialised kernels; everything else with a null factor goes to the general kernel
    if (!d.P1) return false;
    if (!d.P2 && !(d.n2 == 128 && (d.n1 == 32 || d.n1 == 64))) return false;
    if (reinterpret_cast<uintptr_t>(d.P2) & 15) return false;
    const int n1sq = d.n1 * d.n1;
    const uintptr_t a1 = reinterpret_cast<uintptr_t>(d.P1);
    (void)n1sq;
    return (a1 & 3) == 0;
}

int64_t tq_fast_lds_bytes(int n1, int n2) {
    if (n1 < 1 || n1 > kMaxN1 || n2 < 32 || n2 > kMaxN2 || n2 % 32) return 0;
    const int A = (n1 + 31) / 32;
    const int a = variant(A, n2 / 32, n1 % 32 == 0, 0).lds, b = variant(A, n2 / 32, n1 % 32 == 0, 2).lds;
    return a > b ? a : b;
}

hipError_t tq_fast_launch(const TqDev& d, hipStream_t stream) {
    const int A = (d.n1 + 31) / 32, B = d.n2 / 32;
    const bool full1 = (d.n1 % 32) == 0;
    // Kernel flavour (see variant_ab), from measurements on MI355X (tables below): 64-wide rows belong to the
    // wave-per-token kernel except for the smallest launches; when every token can have its own resident workgroup the
    // loop-free kernel wins; of the two persistent loops the pipelined one wins for 32 x 128 from 16384 tokens on and
    // for the other shapes with at most two row tiles, the plain one for 64 x 128 and for three or four row tiles.
    // What the loop-free kernel pays per workgroup is the staging of P1 and P2.  FLATQUANT_MODE overrides the choice
    // for tuning and tests.
    static OccCache occ_cache[4][8][2][5];   // per variant and device
    auto occupancy = [&](int mode, int& occ) -> hipError_t {
        const Variant v = variant(A, B, full1, mode);
        const int threads = mode == 4 ? 64 * kTokensPerWg : 64 * (B / (mode == 1 ? 2 : 1));
        return kernel_occupancy(reinterpret_cast<const void*>(v.fn), threads, v.lds, occ_cache[A - 1][B - 1][full1][mode], occ);
    };
    if (!d.P2) {   // left factor only (n1 = 32 or 64, n2 = 128): loop-free kernel while every token gets a resident workgroup
        {   // wave-per-token kernel (fq_tq_wave.hip), measured against the kernels below (us per launch, cold rotation):
            // 32 x 128: T = 512 4.35 / 4.45, 2048 5.6 / 7.2, 4096 9.0 / 10.8, 8192 15.7 / 17.9, 16384 28.7 / 32.1;
            // 64 x 128: T = 2048 9.6 / 12.1, 8192 35.7 / 32.3, 16384 64.7 / 59.8.  FLATQUANT_MODE = 5 forces it.
            const int m = env_int("FLATQUANT_MODE", -1);
            if ((m == 5 || (m == -1 && d.T > 256 && (d.n1 == 32 || d.T <= 4096))) && po_wave_applicable(d)) return po_wave_launch(d, stream);
        }
        const bool two = (A == 2);
        static OccCache occ_id2[2][2];
        auto kern = [&](int one) -> Variant {
            if (two) return one ? Variant{&tq_fast_kernel<2, 4, 1, true, 2, true>, FastLds<2, 4>::TOTAL} : Variant{&tq_fast_kernel<2, 4, 1, true, 0, true>, FastLds<2, 4>::TOTAL};
            return one ? Variant{&tq_fast_kernel<1, 4, 1, true, 2, true>, FastLds<1, 4>::TOTAL} : Variant{&tq_fast_kernel<1, 4, 1, true, 0, true>, FastLds<1, 4>::TOTAL};
        };
        auto occ_of = [&](int one, int& occ) -> hipError_t {
            const Variant v = kern(one);
            return kernel_occupancy(reinterpret_cast<const void*>(v.fn), 256, v.lds, occ_id2[two][one], occ);
        };
        int occ1 = 0, occ0 = 0;
        hipError_t e = occ_of(1, occ1);
        if (e != hipSuccess) return e;
        int one = (d.T <= (int64_t)cu_count() * occ1) ? 1 : 0;
        const int force = env_int("FLATQUANT_MODE", -1);
        if (force == 0) one = 0;
        if (force == 3 && d.T <= 0x7fffffff) one = 1;
        const Variant v = kern(one);
        int64_t grid = d.T;
        if (!one) {
            e = occ_of(0, occ0);
            if (e != hipSuccess) return e;
            const int64_t resident = (int64_t)cu_count() * occ0;
            const int64_t rounds = (d.T + resident - 1) / resident;
            grid = (d.T + rounds - 1) / rounds;
        }
        return launch(v.fn, dim3((unsigned)grid), dim3(256), v.lds, stream, d, d.clip);
    }
    {   // 64-wide rows (n1 = 32 or 64): the wave-per-token kernel (fq_tq_wave.hip).  Mode 5: one token per wave, the
        // hardware hands out workgroups as earlier ones retire; mode 6: persistent workgroups.  Measured on MI355X
        // (64 x 64, same run, us per launch; loop-free / persistent):
        // T = 2048 6.4 / 7.2, 4096 11.0 / 13.8, 8192 19.9 / 22.6, 16384 35.6 / 40.0, 32768 73.7 / 68.5, 65536 144 / 130,
        // 131072 285 / 254.  Up to 256 tokens the latency of a token's chain of MFMAs is what counts, and the loop-free
        // slab kernel below, which splits a token over two waves, is faster (replayed from a HIP graph, us per launch,
        // wave kernel / slab kernel: T = 64 3.87 / 3.33, 256 4.01 / 3.84, 384 4.15 / 4.60, 512 4.28 / 4.84).
        const int m = env_int("FLATQUANT_MODE", -1);
        if ((m == 5 || m == 6 || (m == -1 && d.T > 256)) && tq_wave_applicable(d))
            return tq_wave_launch(d, stream, env_int("FLATQUANT_WAVE_TPW", 4), m == -1 ? d.T >= 32768 : m == 6, false);
    }
    // 128-wide rows (replayed from a HIP graph up to T = 8192, cold rotation above; us per launch, loop-free / plain
    // loop / pipelined loop): 64 x 128: T = 64 4.2 / 4.4 / 4.9, 512 7.7 / 7.7 / 9.3, 1024 10.5 / 10.7 / 11.4,
    // 2048 17.0 / 15.7 / 16.6, 4096 29.5 / 25.6 / 27.2, 8192 53.5 / 45.2 / 46.7, 16384 - / 75 / 94, 32768 - / 162 / 189;
    // 32 x 128: T = 512 5.4 / 5.4 / 6.6, 1536 10.6 / 8.7 / 9.4, 4096 20.5 / 14.3 / 15.6, 8192 35.8 / 24.5 / 25.6,
    // 16384 - / 41.4 / 38.0.
    int mode = (A <= 2) ? 2 : 0;
    if (A == 2 && (B == 4 || B >= 7)) mode = 0;   // (64 x 256, T = 16384: 226 against 290 us)
    if (A == 1 && B == 4 && d.T <= 8192) mode = 0;
    if (A <= 2 && B == 2 && d.T >= 32768) mode = 1;
    if (A <= 2 && (B <= 2 || B == 4)) {
        int occ3 = 0;
        hipError_t e = occupancy(3, occ3);
        if (e != hipSuccess) return e;
        if (B == 4 ? d.T <= (A == 2 ? 1024 : 512) : d.T <= (int64_t)cu_count() * occ3) mode = 3;
        // past that, and up to where the wave-per-token loop takes over, 64-wide rows do best without a loop as well:
        // workgroups of kTokensPerWg single-wave tokens, handed out by the hardware as earlier ones retire
        // (measured at T = 3072 .. 16384: 3 - 8 % over the pipelined loop)
        else if (B == 2 && d.T < 32768) mode = 4;
    }
    const int mode_env = env_int("FLATQUANT_MODE", -1);
    if (mode_env == 0 || (mode_env == 1 && A <= 2 && (B == 2 || B == 4 || B == 8)) || (mode_env == 2 && A <= 2) || (mode_env == 3 && A <= 2) ||
        (mode_env == 4 && A <= 2 && B == 2)) mode = mode_env;
    const int spw = (mode == 1) ? 2 : 1;
    const Variant v = variant(A, B, full1, mode);
    const int nt = mode == 4 ? 64 * kTokensPerWg : 64 * (B / spw);
    int occ = 0;
    {
        hipError_t e = occupancy(mode, occ);
        if (e != hipSuccess) return e;
    }
    const int cap = env_int("FLATQUANT_WG_PER_CU", 0);
    if (cap > 0 && cap < occ) occ = cap;
    // every workgroup gets the same number of tokens (+-1): grid = ceil(T / ceil(T / resident workgroups))
    const int64_t resident = (int64_t)cu_count() * occ;
    const int64_t rounds = (d.T + resident - 1) / resident;
    int64_t grid = (d.T + rounds - 1) / rounds;
    if (mode >= 3) {
        if (d.T > 0x7fffffff) return hipErrorInvalidConfiguration;   // only reachable through the tuning overrides
        grid = mode == 4 ? (d.T + kTokensPerWg - 1) / kTokensPerWg : d.T;
    }
    return launch(v.fn, dim3((unsigned)grid), dim3(nt), v.lds, stream, d, d.clip);
}

}  // namespace fq
