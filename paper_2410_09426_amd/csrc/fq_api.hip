// C ABI of libflatquant: argument checks, variant selection, launch.  No compute here.
#include "../../include/flatquant.h"
#include "fq_internal.h"

#include <cmath>
#include <utility>
#include <vector>

#include <cstdlib>
#include <cstring>

namespace fq {

static thread_local int g_last_hip_error = 0;

int cu_count() {
    static std::atomic<int> cached[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

hipError_t kernel_occupancy(const void* fn, int threads, int lds, OccCache& cache, int& wg_per_cu) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::atomic<int>* slot = (dev >= 0 && dev < kMaxDevices) ? &cache.per_device[dev] : nullptr;
    int v = slot ? slot->load(std::memory_order_acquire) : 0;
    if (v == 0) {
        e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        int nb = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, fn, threads, lds);
        if (e != hipSuccess) return e;
        if (nb < 1) return hipErrorLaunchOutOfResources;
        v = nb;
        if (slot) slot->store(v, std::memory_order_release);
    }
    wg_per_cu = v;
    return hipSuccess;
}

// Tuning overrides (kernel flavour, workgroups per CU, ...): for measurements and for the tests that must reach every
// code path.  Each starts from the environment variable of the same name, read once per process, and can be changed
// with fq_set_tuning; a launch only reads two atomics per override (no getenv on the launch path).
namespace {
struct Tunable {
    const char* name;
    std::atomic<int> state{0};   // 0: environment not read yet, 1: unset (callers use their default), 2: set
    std::atomic<int> value{0};
    explicit Tunable(const char* n) : name(n) {}
};
Tunable g_tunables[] = {Tunable("FLATQUANT_MODE"), Tunable("FLATQUANT_WG_PER_CU"), Tunable("FLATQUANT_FORCE_GENERIC"),
                        Tunable("FLATQUANT_KV_WG_PER_CU"), Tunable("FLATQUANT_GEMM_TILED"),
                        Tunable("FLATQUANT_GEMM_WIDE"), Tunable("FLATQUANT_GEMM_DEPTH"), Tunable("FLATQUANT_GEMM_WAVES"), Tunable("FLATQUANT_GEMM_ROWS"), Tunable("FLATQUANT_GEMM_RING_MAX_T"), Tunable("FLATQUANT_KV_FOLD_HEADS"), Tunable("FLATQUANT_WAVE_TPW"), Tunable("FLATQUANT_PROBE_SHAPE")};
Tunable* find_tunable(const char* name) {
    for (Tunable& t : g_tunables)
        if (std::strcmp(t.name, name) == 0) return &t;
    return nullptr;
}
}  // namespace

int env_int(const char* name, int dflt) {
    Tunable* t = find_tunable(name);
    if (!t) return dflt;
    int st = t->state.load(std::memory_order_acquire);
    if (st == 0) {   // first use in this process (a second thread doing the same stores the same values)
        const char* v = std::getenv(name);
        if (v && *v) {
            t->value.store(std::atoi(v), std::memory_order_relaxed);
            st = 2;
        } else {
            st = 1;
        }
        int expected = 0;
        if (!t->state.compare_exchange_strong(expected, st, std::memory_order_acq_rel)) st = expected;   // fq_set_tuning came first
    }
    return st == 2 ? t->value.load(std::memory_order_relaxed) : dflt;
}

static fq_status finish(hipError_t e) {
    if (e == hipSuccess) return FQ_OK;
    g_last_hip_error = (int)e;
    return FQ_LAUNCH_FAILED;
}

static bool overlap(const void* a, int64_t na, const void* b, int64_t nb) {
    const char* pa = static_cast<const char*>(a);
    const char* pb = static_cast<const char*>(b);
    return pa < pb + nb && pb < pa + na;
}

}  // namespace fq

extern "C" {

fq_status flatquant_transform_quant(const void* x, const void* P1, const void* P2, const float* clip, int clip_mode,
                                    int64_t T, int n1, int n2, int64_t x_stride, uint8_t* out_codes, void* out_scales,
                                    void* stream) {
    if (T < 0 || n1 < 1 || n2 < 1 || (clip_mode != 0 && clip_mode != 1)) return FQ_INVALID_ARG;
    const int64_t n = (int64_t)n1 * n2;
    if (n % 2 != 0 || x_stride < n) return FQ_INVALID_ARG;
    if (!fq::tq_supported(n1, n2)) return FQ_UNSUPPORTED_SHAPE;
    if (T == 0) return FQ_OK;
    if (!x || !clip || !out_codes || !out_scales) return FQ_INVALID_ARG;   // P1 / P2 may be null: identity
    if ((reinterpret_cast<uintptr_t>(x) & 3) || (x_stride & 1) || (reinterpret_cast<uintptr_t>(P1) & 1) ||
        (reinterpret_cast<uintptr_t>(P2) & 1) || (reinterpret_cast<uintptr_t>(clip) & 3) ||
        (reinterpret_cast<uintptr_t>(out_scales) & 1))
        return FQ_MISALIGNED;
    const int64_t xbytes = ((T - 1) * x_stride + n) * 2;
    if (fq::overlap(x, xbytes, out_codes, T * (n / 2)) || fq::overlap(x, xbytes, out_scales, T * 2) ||
        fq::overlap(out_codes, T * (n / 2), out_scales, T * 2))
        return FQ_INVALID_ARG;
    fq::TqArgs a;
    a.x = static_cast<const _Float16*>(x);
    a.P1 = static_cast<const _Float16*>(P1);
    a.P2 = static_cast<const _Float16*>(P2);
    a.clip = clip; a.clip_mode = clip_mode; a.T = T; a.n1 = n1; a.n2 = n2; a.x_stride = x_stride;
    a.out_codes = out_codes; a.out_scales = static_cast<_Float16*>(out_scales);
    return fq::finish(fq::tq_launch(a, static_cast<hipStream_t>(stream)));
}

static fq_status transform_mxfp4(const void* x, const void* P1, const void* P2, const float* clip, int clip_mode, int64_t T,
                                 int n1, int n2, int64_t x_stride, uint8_t* out_codes, uint8_t* out_scales, void* stream, int tiled);

fq_status flatquant_transform_mxfp4(const void* x, const void* P1, const void* P2, const float* clip, int clip_mode,
                                    int64_t T, int n1, int n2, int64_t x_stride, uint8_t* out_codes, uint8_t* out_scales,
                                    void* stream) {
    return transform_mxfp4(x, P1, P2, clip, clip_mode, T, n1, n2, x_stride, out_codes, out_scales, stream, 0);
}

fq_status flatquant_transform_mxfp4_tiled(const void* x, const void* P1, const void* P2, const float* clip, int clip_mode,
                                          int64_t T, int n1, int n2, int64_t x_stride, uint8_t* out_codes, uint8_t* out_scales,
                                          void* stream) {
    return transform_mxfp4(x, P1, P2, clip, clip_mode, T, n1, n2, x_stride, out_codes, out_scales, stream, 1);
}

int64_t fq_mxfp4_tiled_scale_bytes(int64_t rows, int64_t n) {
    if (rows < 0 || n < 256 || n % 256 != 0) return 0;
    return ((rows + 127) / 128) * 128 * (n / 32);
}

static fq_status transform_mxfp4(const void* x, const void* P1, const void* P2, const float* clip, int clip_mode, int64_t T,
                                 int n1, int n2, int64_t x_stride, uint8_t* out_codes, uint8_t* out_scales, void* stream, int tiled) {
    if (T < 0 || n1 < 1 || n2 < 1 || (clip_mode != 0 && clip_mode != 1)) return FQ_INVALID_ARG;
    const int64_t n = (int64_t)n1 * n2;
    if (x_stride < n) return FQ_INVALID_ARG;
    if (n1 > fq::kMaxN1 || n2 > fq::kMaxN2 || n2 % 2 != 0 || n % 32 != 0) return FQ_UNSUPPORTED_SHAPE;
    if (tiled && n % 256 != 0) return FQ_UNSUPPORTED_SHAPE;
    if (T == 0) return FQ_OK;
    if (!x || !P1 || !P2 || !clip || !out_codes || !out_scales) return FQ_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(x) & 15) || (x_stride & 7) || (reinterpret_cast<uintptr_t>(P1) & 3) ||
        (reinterpret_cast<uintptr_t>(P2) & 15) || (reinterpret_cast<uintptr_t>(clip) & 3) ||
        (reinterpret_cast<uintptr_t>(out_codes) & 15) || (reinterpret_cast<uintptr_t>(out_scales) & (tiled ? 15 : 3)))
        return FQ_MISALIGNED;
    const int64_t xbytes = ((T - 1) * x_stride + n) * 2;
    const int64_t sbytes = tiled ? fq_mxfp4_tiled_scale_bytes(T, n) : T * (n / 32);
    if (fq::overlap(x, xbytes, out_codes, T * (n / 2)) || fq::overlap(x, xbytes, out_scales, sbytes) ||
        fq::overlap(out_codes, T * (n / 2), out_scales, sbytes))
        return FQ_INVALID_ARG;
    fq::TqArgs a;
    a.x = static_cast<const _Float16*>(x);
    a.P1 = static_cast<const _Float16*>(P1);
    a.P2 = static_cast<const _Float16*>(P2);
    a.clip = clip; a.clip_mode = clip_mode; a.T = T; a.n1 = n1; a.n2 = n2; a.x_stride = x_stride;
    a.out_codes = out_codes; a.out_scales = reinterpret_cast<_Float16*>(out_scales);
    a.mx_tiled = tiled;
    const fq::TqDev d = fq::tq_dev_args(a);
    if (fq::tq_mx_applicable(d)) return fq::finish(fq::tq_mx_launch(d, static_cast<hipStream_t>(stream)));
    if (fq::tq_mx_generic_applicable(d)) return fq::finish(fq::tq_mx_generic_launch(d, static_cast<hipStream_t>(stream)));
    return FQ_UNSUPPORTED_SHAPE;
}

fq_status flatquant_weight_transform_quant(const void* w, const void* A1, const void* A2, const float* clip, int clip_mode,
                                           int64_t m, int n1, int n2, int64_t w_stride, uint8_t* out_codes,
                                           void* out_scales, void* stream) {
    // the right factor of Eq. (2) is the left factor's operation on the rows of W with inverse-transposed matrices
    return flatquant_transform_quant(w, A1, A2, clip, clip_mode, m, n1, n2, w_stride, out_codes, out_scales, stream);
}

fq_status flatquant_kv_transform_quant(const void* kv, const void* P, int Hp, float clip, int64_t T, int H, int D,
                                       uint8_t* out_codes, void* out_scales, void* out_zeros, void* stream) {
    return flatquant_kv_transform_quant_bits(kv, P, Hp, clip, 4, T, H, D, out_codes, out_scales, out_zeros, stream);
}

fq_status flatquant_kv_transform_quant_bits(const void* kv, const void* P, int Hp, float clip, int bits, int64_t T, int H, int D,
                                            uint8_t* out_codes, void* out_scales, void* out_zeros, void* stream) {
    if (T < 0 || H < 1 || D < 1 || !(clip > 0.0f)) return FQ_INVALID_ARG;
    if (bits < 2 || bits > 4) return FQ_INVALID_ARG;
    if (Hp != 1 && Hp != H) return FQ_INVALID_ARG;
    if (D != 128 || H > 65535) return FQ_UNSUPPORTED_SHAPE;
    if (T == 0) return FQ_OK;
    if (!kv || !P || !out_codes || !out_scales || !out_zeros) return FQ_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(kv) & 15) || (reinterpret_cast<uintptr_t>(out_codes) & 15) ||
        (reinterpret_cast<uintptr_t>(P) & 1) || (reinterpret_cast<uintptr_t>(out_scales) & 1) ||
        (reinterpret_cast<uintptr_t>(out_zeros) & 1))
        return FQ_MISALIGNED;
    const int64_t g = T * H;
    const int64_t cb = g * D * bits / 8;
    if (fq::overlap(kv, g * D * 2, out_codes, cb) || fq::overlap(kv, g * D * 2, out_scales, g * 2) ||
        fq::overlap(kv, g * D * 2, out_zeros, g * 2) || fq::overlap(out_scales, g * 2, out_zeros, g * 2) ||
        fq::overlap(out_codes, cb, out_scales, g * 2) || fq::overlap(out_codes, cb, out_zeros, g * 2))
        return FQ_INVALID_ARG;
    fq::KvArgs a;
    a.kv = static_cast<const _Float16*>(kv); a.P = static_cast<const _Float16*>(P); a.Hp = Hp; a.clip = clip;
    a.bits = bits;
    a.T = T; a.H = H; a.D = D; a.out_codes = out_codes;
    a.out_scales = static_cast<_Float16*>(out_scales); a.out_zeros = static_cast<_Float16*>(out_zeros);
    return fq::finish(fq::kv_launch(a, static_cast<hipStream_t>(stream)));
}

fq_status flatquant_head_transform(const void* x, const void* P, int Hp, int64_t T, int H, int D, void* out, void* stream) {
    if (T < 0 || H < 1 || D < 1) return FQ_INVALID_ARG;
    if (Hp != 1 && Hp != H) return FQ_INVALID_ARG;
    if (D != 128 || H > 65535) return FQ_UNSUPPORTED_SHAPE;
    if (T == 0) return FQ_OK;
    if (!x || !P || !out) return FQ_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(x) & 15) || (reinterpret_cast<uintptr_t>(out) & 15) || (reinterpret_cast<uintptr_t>(P) & 1))
        return FQ_MISALIGNED;
    const int64_t bytes = T * H * D * 2;
    if (fq::overlap(x, bytes, out, bytes)) return FQ_INVALID_ARG;
    fq::KvArgs a;
    a.kv = static_cast<const _Float16*>(x);
    a.P = static_cast<const _Float16*>(P);
    a.Hp = Hp; a.clip = 1.0f; a.T = T; a.H = H; a.D = D;
    a.out_codes = static_cast<uint8_t*>(out); a.out_scales = nullptr; a.out_zeros = nullptr;
    a.fp16_out = true;
    return fq::finish(fq::kv_launch(a, static_cast<hipStream_t>(stream)));
}

fq_status flatquant_w4a4_gemm(const uint8_t* x_codes, const void* x_scales, const uint8_t* w_codes, const void* w_scales,
                              int64_t T, int m, int n, void* out, int64_t out_stride, void* stream) {
    if (T < 0 || m < 0 || n < 1 || out_stride < m) return FQ_INVALID_ARG;
    if (n % 256 != 0 || n > 65536) return FQ_UNSUPPORTED_SHAPE;
    if (T == 0 || m == 0) return FQ_OK;
    if (!x_codes || !x_scales || !w_codes || !w_scales || !out) return FQ_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(x_codes) & 15) || (reinterpret_cast<uintptr_t>(w_codes) & 15) ||
        (reinterpret_cast<uintptr_t>(x_scales) & 1) || (reinterpret_cast<uintptr_t>(w_scales) & 1) ||
        (reinterpret_cast<uintptr_t>(out) & 1))
        return FQ_MISALIGNED;
    if ((T + 127) / 128 > 0x7fffffffLL || (m + 127) / 128 > 65535) return FQ_UNSUPPORTED_SHAPE;   // grid limits
    const int64_t obytes = ((T - 1) * out_stride + m) * 2;
    if (fq::overlap(x_codes, T * (n / 2), out, obytes) || fq::overlap(w_codes, (int64_t)m * (n / 2), out, obytes) ||
        fq::overlap(x_scales, T * 2, out, obytes) || fq::overlap(w_scales, (int64_t)m * 2, out, obytes))
        return FQ_INVALID_ARG;
    fq::GemmArgs a;
    a.x_codes = x_codes; a.x_scales = static_cast<const _Float16*>(x_scales);
    a.w_codes = w_codes; a.w_scales = static_cast<const _Float16*>(w_scales);
    a.out = static_cast<_Float16*>(out); a.T = T; a.out_stride = out_stride; a.m = m; a.n = n;
    return fq::finish(fq::w4a4_launch(a, static_cast<hipStream_t>(stream)));
}

fq_status flatquant_mxfp4_gemm(const uint8_t* x_codes, const uint8_t* x_scales, const uint8_t* w_codes, const uint8_t* w_scales,
                               int64_t T, int m, int n, void* out, int64_t out_stride, void* stream) {
    if (T < 0 || m < 0 || n < 1 || out_stride < m) return FQ_INVALID_ARG;
    if (n % 256 != 0) return FQ_UNSUPPORTED_SHAPE;
    if (T == 0 || m == 0) return FQ_OK;
    if (!x_codes || !x_scales || !w_codes || !w_scales || !out) return FQ_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(x_codes) & 15) || (reinterpret_cast<uintptr_t>(w_codes) & 15) ||
        (reinterpret_cast<uintptr_t>(x_scales) & 15) || (reinterpret_cast<uintptr_t>(w_scales) & 15) ||
        (reinterpret_cast<uintptr_t>(out) & 1))
        return FQ_MISALIGNED;
    if ((T + 127) / 128 > 0x7fffffffLL || (m + 127) / 128 > 65535) return FQ_UNSUPPORTED_SHAPE;   // grid limits
    const int64_t obytes = ((T - 1) * out_stride + m) * 2;
    if (fq::overlap(x_codes, T * (n / 2), out, obytes) || fq::overlap(w_codes, (int64_t)m * (n / 2), out, obytes) ||
        fq::overlap(x_scales, fq_mxfp4_tiled_scale_bytes(T, n), out, obytes) ||
        fq::overlap(w_scales, fq_mxfp4_tiled_scale_bytes(m, n), out, obytes))
        return FQ_INVALID_ARG;
    fq::MxGemmArgs a;
    a.x_codes = x_codes; a.x_exps = x_scales; a.w_codes = w_codes; a.w_exps = w_scales;
    a.out = static_cast<_Float16*>(out); a.T = T; a.out_stride = out_stride; a.m = m; a.n = n;
    return fq::finish(fq::mxfp4_gemm_launch(a, static_cast<hipStream_t>(stream)));
}

fq_status flatquant_dequant_mxfp4(const uint8_t* codes, const uint8_t* scales, int64_t rows, int n, float* out, void* stream) {
    if (rows < 0 || n < 32 || (n & 31)) return FQ_INVALID_ARG;
    if (rows == 0) return FQ_OK;
    if (!codes || !scales || !out) return FQ_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(codes) & 3) || (reinterpret_cast<uintptr_t>(out) & 3)) return FQ_MISALIGNED;
    return fq::finish(fq::dequant_mxfp4_launch(codes, scales, rows, n, out, static_cast<hipStream_t>(stream)));
}

fq_status flatquant_dequant_bits(const uint8_t* codes, const void* scales, const void* zeros, int64_t rows, int n, int bits,
                                 float* out, void* stream) {
    if (rows < 0 || n < 8 || (n & 7) || bits < 2 || bits > 4) return FQ_INVALID_ARG;
    if (rows == 0) return FQ_OK;
    if (!codes || !scales || !zeros || !out) return FQ_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(scales) & 1) || (reinterpret_cast<uintptr_t>(zeros) & 1) ||
        (reinterpret_cast<uintptr_t>(out) & 3))
        return FQ_MISALIGNED;
    return fq::finish(fq::dequant_bits_launch(codes, static_cast<const _Float16*>(scales), static_cast<const _Float16*>(zeros),
                                              rows, n, bits, out, static_cast<hipStream_t>(stream)));
}

fq_status flatquant_dequant(const uint8_t* codes, const void* scales, const void* zeros, int64_t rows, int n, float* out,
                            void* stream) {
    if (rows < 0 || n < 2 || (n & 1)) return FQ_INVALID_ARG;
    if (rows == 0) return FQ_OK;
    if (!codes || !scales || !out) return FQ_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(scales) & 1) || (reinterpret_cast<uintptr_t>(zeros) & 1) ||
        (reinterpret_cast<uintptr_t>(out) & 3))
        return FQ_MISALIGNED;
    return fq::finish(fq::dequant_launch(codes, static_cast<const _Float16*>(scales), static_cast<const _Float16*>(zeros),
                                         rows, n, out, static_cast<hipStream_t>(stream)));
}

fq_status flatquant_stream_probe(const void* x, int64_t T, int n, int64_t x_stride, uint8_t* out, void* stream) {
    if (T < 0 || n < 32 || x_stride < n) return FQ_INVALID_ARG;
    if (n % 32 != 0) return FQ_UNSUPPORTED_SHAPE;
    if (T == 0) return FQ_OK;
    if (!x || !out) return FQ_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(x) & 15) || (reinterpret_cast<uintptr_t>(out) & 15) || (x_stride & 7)) return FQ_MISALIGNED;
    return fq::finish(fq::stream_probe_launch(x, T, n, x_stride, out, static_cast<hipStream_t>(stream)));
}

int fq_supported(int n1, int n2) { return fq::tq_supported(n1, n2) ? 1 : 0; }

fq_status fq_choose_factors(int64_t n, int* n1, int* n2) {
    if (n < 1 || !n1 || !n2) return FQ_INVALID_ARG;
    int64_t best = 1;
    for (int64_t d = 1; d * d <= n; ++d)
        if (n % d == 0) best = d;
    *n1 = (int)best;
    *n2 = (int)(n / best);
    return FQ_OK;
}

fq_status fq_inverse_transpose(const void* P, int n, void* out, double* max_residual) {
    if (!P || !out || n < 1 || n > 256) return FQ_INVALID_ARG;
    const _Float16* src = static_cast<const _Float16*>(P);
    _Float16* dst = static_cast<_Float16*>(out);
    std::vector<double> a((size_t)n * 2 * n);   // [P | I], reduced to [I | P^-1]
    double big = 0.0;
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) {
            const double v = (double)src[(size_t)i * n + j];
            a[(size_t)i * 2 * n + j] = v;
            a[(size_t)i * 2 * n + n + j] = (i == j) ? 1.0 : 0.0;
            big = std::fmax(big, std::fabs(v));
        }
    if (!(big > 0.0) || !std::isfinite(big)) return FQ_INVALID_ARG;
    for (int col = 0; col < n; ++col) {
        int piv = col;
        for (int r = col + 1; r < n; ++r)
            if (std::fabs(a[(size_t)r * 2 * n + col]) > std::fabs(a[(size_t)piv * 2 * n + col])) piv = r;
        if (!(std::fabs(a[(size_t)piv * 2 * n + col]) > 1e-12 * big)) return FQ_INVALID_ARG;
        if (piv != col)
            for (int j = 0; j < 2 * n; ++j) std::swap(a[(size_t)piv * 2 * n + j], a[(size_t)col * 2 * n + j]);
        const double d = 1.0 / a[(size_t)col * 2 * n + col];
        for (int j = 0; j < 2 * n; ++j) a[(size_t)col * 2 * n + j] *= d;
        for (int r = 0; r < n; ++r) {
            if (r == col) continue;
            const double f = a[(size_t)r * 2 * n + col];
            if (f == 0.0) continue;
            for (int j = 0; j < 2 * n; ++j) a[(size_t)r * 2 * n + j] -= f * a[(size_t)col * 2 * n + j];
        }
    }
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) {
            const double v = a[(size_t)j * 2 * n + n + i];   // transpose of the inverse
            if (!(std::fabs(v) <= 65504.0)) return FQ_INVALID_ARG;
            dst[(size_t)i * n + j] = (_Float16)v;
        }
    if (max_residual) {
        double worst = 0.0;
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) {
                double acc = 0.0;   // (P^T out)[i][j] = sum_k P[k][i] out[k][j]
                for (int k = 0; k < n; ++k) acc += (double)src[(size_t)k * n + i] * (double)dst[(size_t)k * n + j];
                worst = std::fmax(worst, std::fabs(acc - (i == j ? 1.0 : 0.0)));
            }
        *max_residual = worst;
    }
    return FQ_OK;
}

int fq_default_design_fits(int n1, int n2, int64_t m_bytes) {
    if (n1 < 1 || n2 < 1) return 0;
    const int64_t a = ((int64_t)n1 * n1 + 2LL * n1 * n2) * 2;
    const int64_t b = ((int64_t)n2 * n2 + 2LL * n1 * n2) * 2;
    return (a < m_bytes && b < m_bytes) ? 1 : 0;
}

int64_t fq_lds_bytes(int n1, int n2) { return fq::tq_lds_bytes(n1, n2); }

const char* fq_status_string(fq_status s) {
    switch (s) {
        case FQ_OK: return "ok";
        case FQ_INVALID_ARG: return "invalid argument";
        case FQ_UNSUPPORTED_SHAPE: return "unsupported shape";
        case FQ_MISALIGNED: return "misaligned pointer or stride";
        case FQ_LAUNCH_FAILED: return "kernel launch failed";
        default: return "unknown status";
    }
}

int fq_last_hip_error(void) { return fq::g_last_hip_error; }

fq_status fq_set_tuning(const char* name, int value, int enable) {
    if (!name) return FQ_INVALID_ARG;
    fq::Tunable* t = fq::find_tunable(name);
    if (!t) return FQ_INVALID_ARG;
    if (enable) {
        t->value.store(value, std::memory_order_relaxed);
        t->state.store(2, std::memory_order_release);
    } else {
        t->state.store(1, std::memory_order_release);
    }
    return FQ_OK;
}

int fq_abi_version(void) { return 2; }

}  // extern "C"
