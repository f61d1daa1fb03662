// Internal declarations shared by the .hip translation units of libtl.so.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "tl.h"

namespace tl {

// Clang vector types: what the nontemporal and MFMA builtins take.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

// Launchers return hipGetLastError() of their launch.  All pointers are device pointers.
hipError_t launch_unpack2(const uint32_t* packed, int64_t N, int64_t K, int8_t* out, hipStream_t s);
// fx: the fixed-point byte code of Sec. 3.2 (decoded by App. F, Alg. 1) instead of plain base 3
hipError_t launch_unpack3(const uint8_t* packed, int64_t N, int64_t K, int64_t stride, int8_t* out,
                          bool fx, hipStream_t s);
hipError_t launch_probe_copy(void* dst, const void* src, size_t bytes, hipStream_t s);
hipError_t launch_probe_read(const void* src, size_t bytes, void* sink, hipStream_t s);
hipError_t launch_probe_mfma(const __half* x, int64_t x_elems, const uint32_t* Wp, int64_t w_words,
                             int64_t iters, float* sink, double* flops, hipStream_t s);

// Plain VALU kernel: any M, N, K.
hipError_t launch_gemm_generic(const __half* x, const uint32_t* Wp, float gamma, __half* y,
                               int64_t M, int64_t N, int64_t K, hipStream_t s);
hipError_t launch_gemm3_generic(const __half* x, const uint8_t* Wp, int64_t stride, float gamma,
                                __half* y, int64_t M, int64_t N, int64_t K, bool fx, hipStream_t s);

// One GEMM of a grouped call, device pointers, gamma already widened.
struct GemmDesc {
    const __half* x;
    const uint32_t* W;
    __half* y;
    float gamma;
    int64_t M, N, K;
};

// Weight-streaming small-M kernel (2-bit).  Needs K % 64 == 0; handles M in chunks of 16.
bool gemv_supports(int64_t M, int64_t N, int64_t K);
hipError_t launch_gemv(const __half* x, const uint32_t* Wp, float gamma, __half* y,
                       int64_t M, int64_t N, int64_t K, hipStream_t s);
// Whether the small-M kernel takes a GEMM in blocks of 32 activation rows (every decoded weight
// operand feeds two MFMAs) rather than 16.  It halves the passes over W but shortens the items
// (2 tiles instead of 3), which pays when W is large or the blocks are many.  Measured, blocks of
// 32 against blocks of 16 rows (us): 4096 -> 22016 (22.5 MB) M = 17 11.0 / 12.7, M = 64 17.7 / 20.3;
// 4096 -> 14336 (14.7 MB) M = 48 14.5 / 13.7, M = 64 13.7 / 14.2, M = 128 19.0 / 22.2;
// 4096 -> 4096 (4.2 MB) M = 192 13.8 / 13.9, M = 256 13.6 / 14.9; 2048 -> 2048 never.
// Several passes over K (up to 64 slices, 32768): 11008 -> 4096 M = 256 45.1 / 42.7,
// M = 384 59.6 / 65.5; the run of a workgroup must fit its LDS.
inline bool gemv_two_blocks(int64_t M, int64_t N, int64_t K)
{
    const int64_t slices = (K + 511) / 512;
    if (M <= 16 || slices < 2 || slices > 64) return false;
    if (slices > 8) return (N + 15) / 16 <= 256 * 16 && M >= 384;
    const int64_t w_bytes = N * K / 4;
    return w_bytes >= (int64_t(18) << 20) || (M >= 64 && w_bytes >= (int64_t(8) << 20)) ||
           (M >= 256 && w_bytes >= (int64_t(2) << 20));
}

// Several independent GEMMs (each passing gemv_supports) in as few launches as possible.
hipError_t launch_gemv_jobs(const GemmDesc* jobs, int count, hipStream_t s);

// Per-group scales s[K / group][N] in place of gamma (stream form of the small-M kernel; M in
// blocks of 16).  Needs what gemv_supports needs and group % 128 == 0, N % 4 == 0.
bool gemv_gs_supports(int64_t M, int64_t N, int64_t K, int64_t group);
hipError_t launch_gemv_gs(const __half* x, const uint32_t* Wp, const __half* scales, int64_t group,
                          __half* y, int64_t M, int64_t N, int64_t K, hipStream_t s);
// Several such GEMMs (each passing gemv_gs_supports) in as few launches as possible.
struct GemmGsDesc {
    const __half* x;
    const uint32_t* W;
    const __half* scales;
    __half* y;
    int64_t M, N, K, group;
};
hipError_t launch_gemv_gs_jobs(const GemmGsDesc* jobs, int count, hipStream_t s);
// Plain VALU kernel with per-group scales: any M, N, K; group % 16 == 0.
hipError_t launch_gemm_generic_gs(const __half* x, const uint32_t* Wp, const __half* scales,
                                  int64_t group, __half* y, int64_t M, int64_t N, int64_t K,
                                  hipStream_t s);

// Weight-streaming small-M kernel for the 1.6-bit format.  Needs K % 8 == 0.
bool gemv3_supports(int64_t M, int64_t N, int64_t K);
hipError_t launch_gemv3(const __half* x, const uint8_t* Wp, int64_t stride, float gamma, __half* y,
                        int64_t M, int64_t N, int64_t K, bool fx, hipStream_t s);
// Several 1.6-bit GEMMs (each passing gemv3_groups: K in one pass of the stream form) in as few
// launches as possible; all in the same byte code (fx).
struct Gemm3Desc {
    const __half* x;
    const uint8_t* W;
    __half* y;
    float gamma;
    int64_t M, N, K, stride;
};
bool gemv3_groups(int64_t M, int64_t N, int64_t K);
hipError_t launch_gemv3_jobs(const Gemm3Desc* jobs, int count, bool fx, hipStream_t s);

// LDS-tiled MFMA prefill kernel (2-bit).  Needs K % 64 == 0.
bool mfma_supports(int64_t M, int64_t N, int64_t K);
hipError_t launch_mfma(const __half* x, const uint32_t* Wp, float gamma, __half* y,
                       int64_t M, int64_t N, int64_t K, hipStream_t s);

// Prepare every kernel instance on the current device (dynamic-LDS limits); idempotent.
// Once-per-device flags (a function attribute holds for the device it was set on): index of the
// current device, or -1 when it cannot be tracked, in which case the caller does the work again.
constexpr int kMaxDevices = 64;
inline int device_slot()
{
    int d = -1;
    if (hipGetDevice(&d) != hipSuccess) return -1;
    return d >= 0 && d < kMaxDevices ? d : -1;
}

hipError_t gemv_init();
hipError_t gemv3_init();
hipError_t mfma_init();

// fp16 bits -> float on the host (exact).
float half_bits_to_float(uint16_t h);

}  // namespace tl
