// C-ABI entry points that touch the device: argument checks, kernel choice, launch.
#include "tl_internal.hpp"

#include <cmath>

namespace tl {

float half_bits_to_float(uint16_t h)
{
    const int sign = (h >> 15) & 1;
    const int e = (h >> 10) & 0x1F;
    const int f = h & 0x3FF;
    float v;
    if (e == 0) v = std::ldexp(static_cast<float>(f), -24);
    else if (e == 31) v = f ? NAN : INFINITY;
    else v = std::ldexp(static_cast<float>(1024 + f), e - 25);
    return sign ? -v : v;
}

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline bool dims_ok(int64_t M, int64_t N, int64_t K)
{
    const int64_t lim = int64_t(1) << 31;
    return M >= 1 && N >= 1 && K >= 1 && M < lim && N < lim && K < lim &&
           M * N < (int64_t(1) << 40) && N * K < (int64_t(1) << 42) && M * K < (int64_t(1) << 40);
}

inline tl_status from_hip(hipError_t e) { return e == hipSuccess ? TL_OK : TL_ERR_HIP; }

// Most activation rows one launch of the 1.6-bit weight-streaming kernel takes.
constexpr int64_t kGemvMaxM = 4096;

// Small-M kernel (blocks of 16 or 32 activation rows that each stream W) or LDS-tiled MFMA
// kernel, when both can run the shape: whichever the cost models below make cheaper.  They are
// fits to measurements (us; W in MB of packed weights):
//  * small-M, blocks of 32 rows, one pass over K: 4 + blocks x (0.31 + 0.2 W)
//    (4096 -> 14336: 3.2 us per block); several passes: launches of up to 4096 tiles, each
//    passes x (8.7 + 0.88 x its longest run of tiles per workgroup)
//    (11008 -> 4096: 16 blocks 68 us, 8 blocks 47 us)
//  * small-M, blocks of 16 rows: 3.8 + blocks x W x (0.17 while W stays in the L2 caches, 0.21
//    beyond), at least 0.3 per block; when K needs several passes 1 + 3 passes + blocks x 0.175 W
//    (11008 -> 4096: 2 blocks 13.7 us, 16 blocks 44.2 us)
//  * MFMA, 128 x 128 tiles (at most one per CU): 7 + K/64 x (0.43 + 0.09 (tiles - 128)/128 beyond 128
//    tiles) with two sets of waves per tile (K % 128 == 0), else 4 + K/64 x (0.53 + 0.04 tiles/256)
//  * MFMA, 128 x 256 tiles: (5 + K/64 x 0.86) x f(tiles/256), f(r) = 1 up to one tile per CU, then
//    max(r, 0.82 ceil(r)): a round that is not full costs most of a full one
//    (4096 -> 14336: 336 tiles 98 us, 448 tiles 107 us, 896 tiles 219 us).
inline bool prefer_small_m(int64_t M, int64_t N, int64_t K)
{
    if (M <= 16) return true;
    const double w_mb = double(N) * double(K) / 4.0e6;
    const int64_t slices = (K + 511) / 512;
    double t_small;
    if (tl::gemv_two_blocks(M, N, K) && slices > 8) {
        // several passes over K: launches of at most 4096 tiles; a launch costs, per pass, a
        // start plus its longest run of tiles
        const int64_t blocks = (M + 31) / 32, tiles = (N + 15) / 16;
        const int64_t cap = tiles >= 4096 ? 1 : 4096 / tiles;
        const double passes = double((slices + 7) / 8);
        auto launch_us = [&](int64_t b) { return passes * (8.7 + 0.88 * double((b * tiles + 255) / 256)); };
        t_small = double(blocks / cap) * launch_us(cap) + (blocks % cap ? launch_us(blocks % cap) : 0.0);
    } else if (tl::gemv_two_blocks(M, N, K)) {
        t_small = 4.0 + double((M + 31) / 32) * (0.31 + 0.2 * w_mb);
    } else if (slices > 8) {
        t_small = 1.0 + 3.0 * double((slices + 7) / 8) + double((M + 15) / 16) * 0.175 * w_mb;
    } else {
        const double per_mb = w_mb < 8.4 ? 0.17 : 0.21;
        const double per_block = per_mb * w_mb > 0.3 ? per_mb * w_mb : 0.3;
        t_small = 3.8 + double((M + 15) / 16) * per_block;
    }
    const double steps = double(K / 64);
    const double row_blocks = double((M + 127) / 128);
    const double wide = row_blocks * double((N + 255) / 256);
    double t_mfma;
    if (wide <= 128.0) {                                   // 128 x 128 tiles, at most one per CU
        const double tiles = row_blocks * double((N + 127) / 128);
        if (K % 128 == 0)                                  // two sets of waves per tile
            t_mfma = 7.0 + steps * (0.43 + 0.09 * (tiles > 128.0 ? (tiles - 128.0) / 128.0 : 0.0));
        else
            t_mfma = 4.0 + steps * (0.53 + 0.04 * tiles / 256.0);
    } else {                                               // 128 x 256 tiles, in rounds of 256
        const double r = wide / 256.0;
        const double rounds = double(int64_t(r) + (r > double(int64_t(r)) ? 1 : 0));
        const double f = r <= 1.0 ? 1.0 : (r > 0.82 * rounds ? r : 0.82 * rounds);
        t_mfma = (5.0 + steps * 0.86) * f;
    }
    // The constants above were fitted on one machine, and machines differ by several percent
    // (the same library: 18.3 and 19.6 us for the same launch).  Near the crossover the two kernels
    // are within that spread of each other, so a band rather than the bare comparison decides:
    // beyond 16 rows the tiled kernel takes the shape unless the model puts the small-M kernel
    // ahead by more than 5 %.
    return 1.05 * t_small < t_mfma;
}

}  // namespace
}  // namespace tl

extern "C" {

tl_status tl_unpack_dev(tl_format fmt, const void* packed, int64_t N, int64_t K, int8_t* W_out,
                        void* stream)
{
    if (!packed || !W_out) return TL_ERR_NULL;
    if (!tl::dims_ok(1, N, K)) return TL_ERR_SHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (fmt == TL_FMT_2BIT)
        return tl::from_hip(tl::launch_unpack2(static_cast<const uint32_t*>(packed), N, K, W_out, s));
    if (fmt == TL_FMT_1P6BIT || fmt == TL_FMT_1P6BIT_FX)
        return tl::from_hip(tl::launch_unpack3(static_cast<const uint8_t*>(packed), N, K,
                                               static_cast<int64_t>(tl_row_stride_bytes(fmt, K)),
                                               W_out, fmt == TL_FMT_1P6BIT_FX, s));
    return TL_ERR_UNSUPPORTED;
}

tl_path tl_ternary_gemm_which(int64_t M, int64_t N, int64_t K)
{
    if (!tl::dims_ok(M, N, K)) return TL_PATH_AUTO;
    if (tl::gemv_supports(M, N, K) && (tl::prefer_small_m(M, N, K) || !tl::mfma_supports(M, N, K))) return TL_PATH_GEMV;
    if (tl::mfma_supports(M, N, K)) return TL_PATH_MFMA;
    return TL_PATH_GENERIC;
}

tl_status tl_ternary_gemm_path(const void* x, const void* Wpacked, uint16_t gamma_fp16_bits, void* y,
                               int64_t M, int64_t N, int64_t K, void* stream, tl_path path)
{
    if (!x || !Wpacked || !y) return TL_ERR_NULL;
    if (!tl::dims_ok(M, N, K)) return TL_ERR_SHAPE;
    if (!tl::aligned16(x) || !tl::aligned16(Wpacked) || !tl::aligned16(y)) return TL_ERR_ALIGN;
    const float gamma = tl::half_bits_to_float(gamma_fp16_bits);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const __half* xh = static_cast<const __half*>(x);
    const uint32_t* wp = static_cast<const uint32_t*>(Wpacked);
    __half* yh = static_cast<__half*>(y);

    if (path == TL_PATH_AUTO) path = tl_ternary_gemm_which(M, N, K);
    switch (path) {
        case TL_PATH_GENERIC:
            return tl::from_hip(tl::launch_gemm_generic(xh, wp, gamma, yh, M, N, K, s));
        case TL_PATH_GEMV:
            if (!tl::gemv_supports(M, N, K)) return TL_ERR_UNSUPPORTED;
            return tl::from_hip(tl::launch_gemv(xh, wp, gamma, yh, M, N, K, s));
        case TL_PATH_MFMA:
            if (!tl::mfma_supports(M, N, K)) return TL_ERR_UNSUPPORTED;
            return tl::from_hip(tl::launch_mfma(xh, wp, gamma, yh, M, N, K, s));
        default:
            return TL_ERR_UNSUPPORTED;
    }
}

tl_status tl_ternary_gemm(const void* x, const void* Wpacked, uint16_t gamma_fp16_bits, void* y,
                          int64_t M, int64_t N, int64_t K, void* stream)
{
    return tl_ternary_gemm_path(x, Wpacked, gamma_fp16_bits, y, M, N, K, stream, TL_PATH_AUTO);
}

tl_status tl_ternary_gemm_grouped(const tl_gemm_job* jobs, int64_t count, void* stream)
{
    if (count == 0) return TL_OK;
    if (!jobs) return TL_ERR_NULL;
    if (count < 0 || count > 4096) return TL_ERR_SHAPE;
    for (int64_t i = 0; i < count; ++i) {
        const tl_gemm_job& j = jobs[i];
        if (!j.x || !j.Wpacked || !j.y) return TL_ERR_NULL;
        if (!tl::dims_ok(j.M, j.N, j.K)) return TL_ERR_SHAPE;
        if (!tl::aligned16(j.x) || !tl::aligned16(j.Wpacked) || !tl::aligned16(j.y)) return TL_ERR_ALIGN;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    // Jobs the small-M kernel takes are fused; the others go through tl_ternary_gemm one by one.
    tl::GemmDesc fused[64];
    int nf = 0;
    auto flush = [&]() -> tl_status {
        if (nf == 0) return TL_OK;
        const hipError_t e = tl::launch_gemv_jobs(fused, nf, s);
        nf = 0;
        return tl::from_hip(e);
    };
    for (int64_t i = 0; i < count; ++i) {
        const tl_gemm_job& j = jobs[i];
        if (tl_ternary_gemm_which(j.M, j.N, j.K) == TL_PATH_GEMV) {
            fused[nf++] = tl::GemmDesc{static_cast<const __half*>(j.x), static_cast<const uint32_t*>(j.Wpacked),
                                       static_cast<__half*>(j.y), tl::half_bits_to_float(j.gamma_fp16_bits),
                                       j.M, j.N, j.K};
            if (nf == 64) { const tl_status st = flush(); if (st != TL_OK) return st; }
        } else {
            tl_status st = flush();
            if (st != TL_OK) return st;
            st = tl_ternary_gemm(j.x, j.Wpacked, j.gamma_fp16_bits, j.y, j.M, j.N, j.K, stream);
            if (st != TL_OK) return st;
        }
    }
    return flush();
}

namespace {

tl_status gemm_1p6(const void* x, const void* Wpacked, uint16_t gamma_fp16_bits, void* y,
                   int64_t M, int64_t N, int64_t K, void* stream, bool fx)
{
    if (!x || !Wpacked || !y) return TL_ERR_NULL;
    if (!tl::dims_ok(M, N, K)) return TL_ERR_SHAPE;
    if (!tl::aligned16(x) || !tl::aligned16(Wpacked) || !tl::aligned16(y)) return TL_ERR_ALIGN;
    const float gamma = tl::half_bits_to_float(gamma_fp16_bits);
    const int64_t stride = static_cast<int64_t>(tl_row_stride_bytes(TL_FMT_1P6BIT, K));
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (tl::gemv3_supports(M < tl::kGemvMaxM ? M : tl::kGemvMaxM, N, K)) {
        // more rows than one launch takes: one launch per kGemvMaxM rows
        const __half* xh = static_cast<const __half*>(x);
        __half* yh = static_cast<__half*>(y);
        for (int64_t m0 = 0; m0 < M; m0 += tl::kGemvMaxM) {
            const int64_t rows = M - m0 < tl::kGemvMaxM ? M - m0 : tl::kGemvMaxM;
            const hipError_t e = tl::launch_gemv3(xh + m0 * K, static_cast<const uint8_t*>(Wpacked), stride, gamma,
                                                  yh + m0 * N, rows, N, K, fx, s);
            if (e != hipSuccess) return tl::from_hip(e);
        }
        return TL_OK;
    }
    return tl::from_hip(tl::launch_gemm3_generic(static_cast<const __half*>(x),
                                                 static_cast<const uint8_t*>(Wpacked), stride, gamma,
                                                 static_cast<__half*>(y), M, N, K, fx, s));
}

}  // namespace

tl_status tl_ternary_gemm_1p6(const void* x, const void* Wpacked, uint16_t gamma_fp16_bits, void* y,
                              int64_t M, int64_t N, int64_t K, void* stream)
{
    return gemm_1p6(x, Wpacked, gamma_fp16_bits, y, M, N, K, stream, false);
}

tl_status tl_ternary_gemm_1p6_fx(const void* x, const void* Wpacked, uint16_t gamma_fp16_bits, void* y,
                                 int64_t M, int64_t N, int64_t K, void* stream)
{
    return gemm_1p6(x, Wpacked, gamma_fp16_bits, y, M, N, K, stream, true);
}

tl_status tl_ternary_gemm_gs(const void* x, const void* Wpacked, const void* scales, int64_t group,
                             void* y, int64_t M, int64_t N, int64_t K, void* stream)
{
    if (!x || !Wpacked || !scales || !y) return TL_ERR_NULL;
    if (!tl::dims_ok(M, N, K)) return TL_ERR_SHAPE;
    if (group < 16 || group % 16 != 0) return TL_ERR_SHAPE;
    if (!tl::aligned16(x) || !tl::aligned16(Wpacked) || !tl::aligned16(scales) || !tl::aligned16(y)) return TL_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const __half* xh = static_cast<const __half*>(x);
    const uint32_t* wp = static_cast<const uint32_t*>(Wpacked);
    const __half* sh = static_cast<const __half*>(scales);
    __half* yh = static_cast<__half*>(y);
    if (tl::gemv_gs_supports(M, N, K, group)) {
        const hipError_t e = tl::launch_gemv_gs(xh, wp, sh, group, yh, M, N, K, s);
        if (e != hipErrorInvalidValue) return tl::from_hip(e);
        (void)hipGetLastError();                 // nothing was launched: the plain kernel takes it
    }
    return tl::from_hip(tl::launch_gemm_generic_gs(xh, wp, sh, group, yh, M, N, K, s));
}

tl_status tl_ternary_gemm_1p6_grouped(const tl_gemm_job* jobs, int64_t count, tl_format format, void* stream)
{
    if (count == 0) return TL_OK;
    if (!jobs) return TL_ERR_NULL;
    if (count < 0 || count > 4096) return TL_ERR_SHAPE;
    if (format != TL_FMT_1P6BIT && format != TL_FMT_1P6BIT_FX) return TL_ERR_VALUE;
    for (int64_t i = 0; i < count; ++i) {
        const tl_gemm_job& j = jobs[i];
        if (!j.x || !j.Wpacked || !j.y) return TL_ERR_NULL;
        if (!tl::dims_ok(j.M, j.N, j.K)) return TL_ERR_SHAPE;
        if (!tl::aligned16(j.x) || !tl::aligned16(j.Wpacked) || !tl::aligned16(j.y)) return TL_ERR_ALIGN;
    }
    const bool fx = format == TL_FMT_1P6BIT_FX;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // Jobs whose K fits one pass of the stream form share launches; the others go one by one.
    tl::Gemm3Desc fused[64];
    int nf = 0;
    auto flush = [&]() -> tl_status {
        if (nf == 0) return TL_OK;
        const hipError_t e = tl::launch_gemv3_jobs(fused, nf, fx, s);
        nf = 0;
        return tl::from_hip(e);
    };
    for (int64_t i = 0; i < count; ++i) {
        const tl_gemm_job& j = jobs[i];
        if (tl::gemv3_groups(j.M, j.N, j.K)) {
            fused[nf++] = tl::Gemm3Desc{static_cast<const __half*>(j.x), static_cast<const uint8_t*>(j.Wpacked),
                                        static_cast<__half*>(j.y), tl::half_bits_to_float(j.gamma_fp16_bits),
                                        j.M, j.N, j.K, static_cast<int64_t>(tl_row_stride_bytes(TL_FMT_1P6BIT, j.K))};
            if (nf == 64) { const tl_status st = flush(); if (st != TL_OK) return st; }
        } else {
            const tl_status st = gemm_1p6(j.x, j.Wpacked, j.gamma_fp16_bits, j.y, j.M, j.N, j.K, stream, fx);
            if (st != TL_OK) return st;
        }
    }
    return flush();
}

tl_status tl_ternary_gemm_gs_grouped(const tl_gemm_gs_job* jobs, int64_t count, void* stream)
{
    if (count == 0) return TL_OK;
    if (!jobs) return TL_ERR_NULL;
    if (count < 0 || count > 4096) return TL_ERR_SHAPE;
    for (int64_t i = 0; i < count; ++i) {
        const tl_gemm_gs_job& j = jobs[i];
        if (!j.x || !j.Wpacked || !j.scales || !j.y) return TL_ERR_NULL;
        if (!tl::dims_ok(j.M, j.N, j.K)) return TL_ERR_SHAPE;
        if (j.group < 16 || j.group % 16 != 0) return TL_ERR_SHAPE;
        if (!tl::aligned16(j.x) || !tl::aligned16(j.Wpacked) || !tl::aligned16(j.scales) || !tl::aligned16(j.y)) return TL_ERR_ALIGN;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    // Jobs the weight-streaming kernel takes share launches; the others go one by one.
    tl::GemmGsDesc fused[64];
    int nf = 0;
    auto flush = [&]() -> tl_status {
        if (nf == 0) return TL_OK;
        const hipError_t e = tl::launch_gemv_gs_jobs(fused, nf, s);
        nf = 0;
        return tl::from_hip(e);
    };
    for (int64_t i = 0; i < count; ++i) {
        const tl_gemm_gs_job& j = jobs[i];
        if (tl::gemv_gs_supports(j.M, j.N, j.K, j.group)) {
            fused[nf++] = tl::GemmGsDesc{static_cast<const __half*>(j.x), static_cast<const uint32_t*>(j.Wpacked),
                                         static_cast<const __half*>(j.scales), static_cast<__half*>(j.y),
                                         j.M, j.N, j.K, j.group};
            if (nf == 64) { const tl_status st = flush(); if (st != TL_OK) return st; }
        } else {
            const tl_status st = tl_ternary_gemm_gs(j.x, j.Wpacked, j.scales, j.group, j.y, j.M, j.N, j.K, stream);
            if (st != TL_OK) return st;
        }
    }
    return flush();
}

tl_status tl_init(void)
{
    hipError_t e = tl::gemv_init();
    if (e == hipSuccess) e = tl::gemv3_init();
    if (e == hipSuccess) e = tl::mfma_init();
    return tl::from_hip(e);
}

tl_status tl_probe_copy(void* dst, const void* src, size_t bytes, void* stream)
{
    if (!dst || !src) return TL_ERR_NULL;
    if (bytes % 16 != 0) return TL_ERR_SHAPE;
    if (!tl::aligned16(dst) || !tl::aligned16(src)) return TL_ERR_ALIGN;
    return tl::from_hip(tl::launch_probe_copy(dst, src, bytes, static_cast<hipStream_t>(stream)));
}

tl_status tl_probe_read(const void* src, size_t bytes, void* sink, void* stream)
{
    if (!src || !sink) return TL_ERR_NULL;
    if (bytes % 16 != 0) return TL_ERR_SHAPE;
    if (!tl::aligned16(src) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return TL_ERR_ALIGN;
    return tl::from_hip(tl::launch_probe_read(src, bytes, sink, static_cast<hipStream_t>(stream)));
}

tl_status tl_probe_mfma(const void* x, int64_t x_elems, const void* Wpacked, int64_t w_words, int64_t iters,
                        void* sink, double* flops, void* stream)
{
    if (!x || !Wpacked || !sink) return TL_ERR_NULL;
    if (x_elems < 1 || w_words < 1 || iters < 1 || iters > (int64_t(1) << 24)) return TL_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(x) & 1u) || (reinterpret_cast<uintptr_t>(Wpacked) & 3u) ||
        (reinterpret_cast<uintptr_t>(sink) & 3u)) return TL_ERR_ALIGN;
    return tl::from_hip(tl::launch_probe_mfma(static_cast<const __half*>(x), x_elems, static_cast<const uint32_t*>(Wpacked),
                                              w_words, iters, static_cast<float*>(sink), flops, static_cast<hipStream_t>(stream)));
}

}  // extern "C"
