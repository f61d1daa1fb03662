// Device decode (byte-exact twin of the host decoders), the measurement probes (copy, read-only,
// bare MFMA loop) and the generic VALU GEMMs that accept every shape.
#include "tl_internal.hpp"

namespace tl {

namespace {

// ---- Sec. 3.1 decode: one thread per 32-bit word, 16 weights out -------------------
__global__ void __launch_bounds__(256)
unpack2_kernel(const uint32_t* __restrict__ packed, int64_t N, int64_t K, int64_t words,
               int8_t* __restrict__ out)
{
    const int64_t gid = blockIdx.x * int64_t(256) + threadIdx.x;
    if (gid >= N * words) return;
    const int64_t n = gid / words;
    const int64_t i = gid - n * words;
    uint32_t word = packed[gid];
    const int64_t base = 16 * i;
    int8_t* dst = out + n * K + base;
    const int len = (K - base < 16) ? int(K - base) : 16;
    for (int j = 0; j < len; ++j, word >>= 2) dst[j] = int8_t(int(word & 3u) - 1);
}

// Digit i (0..4) of a 1.6-bit byte as w + 1.  Plain form: base-3 digits, least significant
// first.  Fixed-point form (Sec. 3.2 with k = 5, p = 8): the byte is b = ceil(256 V / 243) for the
// block value V = sum_j d_j 3^(4-j) < 243, so V = floor(243 b / 256) gives it back, and its base-3
// digits are taken most significant first.  (The multiply-by-3 peeling of App. F, Alg. 1 yields
// the same digits for every byte; the tests check this decode against it.)
__device__ __forceinline__ void digits5(unsigned v, bool fx, unsigned (&d)[5])
{
    if (fx) {
        v = (v * 243u) >> 8;
#pragma unroll
        for (int i = 4; i >= 0; --i) {
            const unsigned q = v / 3u;
            d[i] = v - 3u * q;
            v = q;
        }
    } else {
        v = (v >= 243u) ? v - 243u : v;
#pragma unroll
        for (int i = 0; i < 5; ++i) {
            const unsigned q = v / 3u;
            d[i] = v - 3u * q;
            v = q;
        }
    }
}

// ---- base-3 byte decode: one thread per byte, up to 5 weights out ------------------
__global__ void __launch_bounds__(256)
unpack3_kernel(const uint8_t* __restrict__ packed, int64_t N, int64_t K, int64_t stride,
               int64_t nbytes, int8_t* __restrict__ out, bool fx)
{
    const int64_t gid = blockIdx.x * int64_t(256) + threadIdx.x;
    if (gid >= N * nbytes) return;
    const int64_t n = gid / nbytes;
    const int64_t b = gid - n * nbytes;
    unsigned d[5];
    digits5(packed[n * stride + b], fx, d);
    const int64_t base = 5 * b;
    int8_t* dst = out + n * K + base;
#pragma unroll
    for (int i = 0; i < 5; ++i)
        if (base + i < K) dst[i] = int8_t(int(d[i]) - 1);
}

__global__ void __launch_bounds__(256)
probe_copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src, size_t n16)
{
    size_t i = blockIdx.x * size_t(256) + threadIdx.x;
    const size_t step = size_t(gridDim.x) * 256;
    for (; i < n16; i += step) dst[i] = __builtin_nontemporal_load(src + i);
}

// Streaming read with nothing else: every workgroup requests its 16 KB (four 16-byte loads
// per thread, all in flight together) and exits; workgroups are as many as the buffer needs,
// so the dispatcher walks the buffer front to back.  The words are folded together and stored
// only if the fold equals a value it practically never has, which keeps the loads alive.
__global__ void __launch_bounds__(256)
probe_read_kernel(const u32x4* __restrict__ src, size_t n16, unsigned* __restrict__ sink)
{
    typedef const __attribute__((address_space(1))) u32x4* gptr;
    const size_t base = size_t(blockIdx.x) * 1024 + threadIdx.x;
    u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const size_t i = base + size_t(u) * 256;
        v[u] = i < n16 ? __builtin_nontemporal_load((gptr)(src + i)) : u32x4{0u, 0u, 0u, 0u};
    }
    unsigned acc = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    if (acc == 0x9E3779B9u) *sink = acc;
}

// ---- generic GEMM ---------------------------------------------------------------
// Takes every shape (any K: packed rows and activation rows may start at any word / any even
// byte).  A workgroup of 4 waves computes 16 activation rows x 16 output rows and walks K in
// chunks of 1024.  The chunk's activations are staged in LDS as fp16 with coalesced 4-byte
// (K even) or 2-byte loads, zero past K, so a code beyond K meets a zero.  Wave w
// owns output rows 4w .. 4w+3: lane l decodes word l of the chunk of each of them with
// shift-and-mask exactly as Sec. 3.1 states it (w = code - 1), reads its 16 activations of a
// row from LDS and accumulates w x in fp32; the lanes' sums are folded across the wave at the end.
constexpr int MB = 4;                  // activation rows per workgroup of the other generic kernels
constexpr int GM = 16;                 // activation rows per workgroup
constexpr int GN = 16;                 // output rows per workgroup (4 per wave)
constexpr int GKC = 1024;              // K per chunk: one packed word per lane
constexpr int GROW = GKC + 8;          // halves per staged row (16 bytes of padding)

__device__ __forceinline__ float wave_sum(float v)
{
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// GS: one fp16 scale per `group` weights along K and output row, s[K / group][N] (group % 16 == 0,
// so a packed word lies inside one group), instead of gamma: the word's weights are scaled as
// they are decoded (s w is exact), y = fp16(sum).
template <bool GS>
__global__ void __launch_bounds__(256)
gemm_generic_kernel(const __half* __restrict__ x, const uint32_t* __restrict__ Wp, float gamma,
                    const __half* __restrict__ scales, int64_t group,
                    __half* __restrict__ y, int64_t M, int64_t N, int64_t K, int64_t words)
{
    __shared__ __attribute__((aligned(16))) __half xs[GM * GROW];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int64_t n0 = blockIdx.x * int64_t(GN) + wave * 4;
    const int64_t m0 = blockIdx.y * int64_t(GM);
    const int mrem = int(M - m0 < GM ? M - m0 : GM);
    float acc[GM][4];
#pragma unroll
    for (int r = 0; r < GM; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[r][c] = 0.f;

    for (int64_t kc = 0; kc < K; kc += GKC) {
        // this chunk's packed words first: they travel while the activations are staged
        const int64_t i = kc / 16 + lane;
        uint32_t word[4];
        float sc[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int64_t n = n0 + c;
            word[c] = 0x55555555u;                     // all codes 1: weights 0
            sc[c] = GS ? 0.f : 1.f;
            if (n < N && i < words) {
                word[c] = Wp[n * words + i];
                if constexpr (GS) sc[c] = __half2float(scales[((16 * i) / group) * N + n]);
            }
        }
        __syncthreads();                               // the chunk before has been consumed
        // rows that exist only; 8 loads in flight per thread
        if ((K & 1) == 0) {
            const int total = mrem * (GKC / 2);
            for (int base = tid; base < total; base += 256 * 8) {
                uint32_t v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int idx = base + u * 256;
                    const int r = idx / (GKC / 2);
                    const int kp = (idx - r * (GKC / 2)) * 2;
                    v[u] = 0u;
                    if (idx < total && kc + kp < K)    // K and kp even: the pair lies inside the row
                        v[u] = *reinterpret_cast<const uint32_t*>(x + (m0 + r) * K + kc + kp);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int idx = base + u * 256;
                    const int r = idx / (GKC / 2);
                    const int kp = (idx - r * (GKC / 2)) * 2;
                    if (idx < total) *reinterpret_cast<uint32_t*>(xs + r * GROW + kp) = v[u];
                }
            }
        } else {
            const int total = mrem * GKC;
            for (int base = tid; base < total; base += 256 * 8) {
                __half v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int idx = base + u * 256;
                    const int r = idx / GKC;
                    const int k = idx - r * GKC;
                    v[u] = __ushort_as_half(0);
                    if (idx < total && kc + k < K) v[u] = x[(m0 + r) * K + kc + k];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int idx = base + u * 256;
                    const int r = idx / GKC;
                    const int k = idx - r * GKC;
                    if (idx < total) xs[r * GROW + k] = v[u];
                }
            }
        }
        __syncthreads();

        float wf[4][16];
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const float w = float(int((word[c] >> (2 * j)) & 3u) - 1);
                wf[c][j] = GS ? sc[c] * w : w;
            }
#pragma unroll
        for (int r = 0; r < GM; ++r) {
            if (r < mrem) {
                const f16x8 lo = *reinterpret_cast<const f16x8*>(xs + r * GROW + 16 * lane);
                const f16x8 hi = *reinterpret_cast<const f16x8*>(xs + r * GROW + 16 * lane + 8);
                float xf[16];
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    xf[q] = float(lo[q]);
                    xf[8 + q] = float(hi[q]);
                }
#pragma unroll
                for (int c = 0; c < 4; ++c)
#pragma unroll
                    for (int j = 0; j < 16; ++j) acc[r][c] = fmaf(wf[c][j], xf[j], acc[r][c]);
            }
        }
    }
    // Fold the 64 sums of every lane across the wave: each butterfly step halves the values a
    // lane carries (it keeps the half its lane bit selects and adds the partner's copy of it), so
    // after 6 steps lane l holds the total of sum number l = 4 r + c.
    float v[GM * 4];
#pragma unroll
    for (int r = 0; r < GM; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) v[4 * r + c] = acc[r][c];
#pragma unroll
    for (int half = 32; half >= 1; half >>= 1) {
        const bool upper = (lane & half) != 0;
#pragma unroll
        for (int q = 0; q < half; ++q) {
            const float send = upper ? v[q] : v[q + half];
            const float keep = upper ? v[q + half] : v[q];
            v[q] = keep + __shfl_xor(send, half, 64);
        }
    }
    const int r = lane >> 2, c = lane & 3;
    if (r < mrem && n0 + c < N) y[(m0 + r) * N + n0 + c] = __float2half_rn(GS ? v[0] : gamma * v[0]);
}

__global__ void __launch_bounds__(256)
gemm3_generic_kernel(const __half* __restrict__ x, const uint8_t* __restrict__ Wp, int64_t stride,
                     float gamma, __half* __restrict__ y, int64_t M, int64_t N, int64_t K, bool fx)
{
    const int lane = threadIdx.x & 63;
    const int64_t n = blockIdx.x * int64_t(4) + (threadIdx.x >> 6);
    const int64_t m0 = blockIdx.y * int64_t(MB);
    if (n >= N) return;
    float acc[MB];
    for (int r = 0; r < MB; ++r) acc[r] = 0.f;
    const uint8_t* row = Wp + n * stride;
    const int64_t nbytes = (K + 4) / 5;
    for (int64_t b = lane; b < nbytes; b += 64) {
        unsigned d[5];
        digits5(row[b], fx, d);
        const int64_t base = 5 * b;
        for (int i = 0; i < 5 && base + i < K; ++i) {
            const int w = int(d[i]) - 1;
            for (int r = 0; r < MB; ++r) {
                if (m0 + r < M) {
                    const float xv = __half2float(x[(m0 + r) * K + base + i]);
                    acc[r] += (w > 0) ? xv : ((w < 0) ? -xv : 0.f);
                }
            }
        }
    }
    for (int r = 0; r < MB; ++r) {
        const float s = wave_sum(acc[r]);
        if (lane == 0 && m0 + r < M) y[(m0 + r) * N + n] = __float2half_rn(gamma * s);
    }
}

// ---- matrix-pipe ceiling: waves that only issue v_mfma_f32_32x32x16_f16 -----------------------
// 8 independent accumulators per wave, two waves per SIMD (256 workgroups of 8 waves), no memory,
// LDS or vector-ALU work inside the loop.  The operands are real data, because the data decides
// what the chip can sustain: one operand holds activations as they are, the other ternary weights
// decoded to fp16 -1 / 0 / +1 from packed words (Sec. 3.1), as the large-M kernel feeds them.
constexpr int kProbeMfmaGroups = 256, kProbeMfmaThreads = 512, kProbeMfmaAcc = 8;

__global__ void __launch_bounds__(kProbeMfmaThreads)
probe_mfma_kernel(const __half* __restrict__ x, int64_t x_elems, const uint32_t* __restrict__ Wp, int64_t w_words,
                  int64_t iters, float* __restrict__ sink)
{
    const int64_t t = int64_t(blockIdx.x) * kProbeMfmaThreads + threadIdx.x;
    f16x8 a[2], b[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const uint32_t word = Wp[(2 * t + q) % w_words];          // 16 codes; 8 of them are used
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            a[q][e] = static_cast<_Float16>(__half2float(x[((2 * t + q) * 8 + e) % x_elems]));
            int c = int((word >> (2 * e)) & 3u);
            if (c == 3) c = 1;                                    // (never packed) counts as weight 0
            b[q][e] = static_cast<_Float16>(float(c - 1));
        }
    }
    f32x16 acc[kProbeMfmaAcc];
#pragma unroll
    for (int q = 0; q < kProbeMfmaAcc; ++q)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[q][r] = 0.f;
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int q = 0; q < kProbeMfmaAcc; ++q)
            acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[q & 1], b[(q >> 1) & 1], acc[q], 0, 0, 0);
    }
    float fold = 0.f;
#pragma unroll
    for (int q = 0; q < kProbeMfmaAcc; ++q)
#pragma unroll
        for (int r = 0; r < 16; ++r) fold += acc[q][r];
    if (fold == 1.2345678e30f) sink[0] = fold;                    // keeps the loop alive
}

inline unsigned blocks_for(int64_t items, int per_block)
{
    return static_cast<unsigned>((items + per_block - 1) / per_block);
}

}  // namespace

hipError_t launch_unpack2(const uint32_t* packed, int64_t N, int64_t K, int8_t* out, hipStream_t s)
{
    const int64_t words = (K + 15) / 16;
    hipLaunchKernelGGL(unpack2_kernel, dim3(blocks_for(N * words, 256)), dim3(256), 0, s,
                       packed, N, K, words, out);
    return hipGetLastError();
}

hipError_t launch_unpack3(const uint8_t* packed, int64_t N, int64_t K, int64_t stride, int8_t* out,
                          bool fx, hipStream_t s)
{
    const int64_t nbytes = (K + 4) / 5;
    hipLaunchKernelGGL(unpack3_kernel, dim3(blocks_for(N * nbytes, 256)), dim3(256), 0, s,
                       packed, N, K, stride, nbytes, out, fx);
    return hipGetLastError();
}

hipError_t launch_probe_copy(void* dst, const void* src, size_t bytes, hipStream_t s)
{
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(probe_copy_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s,
                       static_cast<u32x4*>(dst), static_cast<const u32x4*>(src), n16);
    return hipGetLastError();
}

hipError_t launch_probe_mfma(const __half* x, int64_t x_elems, const uint32_t* Wp, int64_t w_words,
                             int64_t iters, float* sink, double* flops, hipStream_t s)
{
    if (flops) *flops = double(kProbeMfmaGroups) * (kProbeMfmaThreads / 64) * double(iters) * kProbeMfmaAcc * (2.0 * 32 * 32 * 16);
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(kProbeMfmaGroups), dim3(kProbeMfmaThreads), 0, s, x, x_elems, Wp, w_words, iters, sink);
    return hipGetLastError();
}

hipError_t launch_probe_read(const void* src, size_t bytes, void* sink, hipStream_t s)
{
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    const size_t blocks = (n16 + 1023) / 1024;
    if (blocks > 0x7fffffffu) return hipErrorInvalidValue;
    hipLaunchKernelGGL(probe_read_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s,
                       static_cast<const u32x4*>(src), n16, static_cast<unsigned*>(sink));
    return hipGetLastError();
}

// The row blocks of these kernels lie on grid.y, which holds 65535 of them: more activation rows go
// out as several launches.
constexpr int64_t kMaxGridY = 65535;

hipError_t launch_gemm_generic(const __half* x, const uint32_t* Wp, float gamma, __half* y,
                               int64_t M, int64_t N, int64_t K, hipStream_t s)
{
    const int64_t words = (K + 15) / 16;
    for (int64_t m0 = 0; m0 < M; m0 += kMaxGridY * GM) {
        const int64_t rows = M - m0 < kMaxGridY * GM ? M - m0 : kMaxGridY * GM;
        dim3 grid(blocks_for(N, GN), blocks_for(rows, GM));
        hipLaunchKernelGGL(gemm_generic_kernel<false>, grid, dim3(256), 0, s, x + m0 * K, Wp, gamma,
                           static_cast<const __half*>(nullptr), int64_t(16), y + m0 * N, rows, N, K, words);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_gemm_generic_gs(const __half* x, const uint32_t* Wp, const __half* scales,
                                  int64_t group, __half* y, int64_t M, int64_t N, int64_t K,
                                  hipStream_t s)
{
    const int64_t words = (K + 15) / 16;
    for (int64_t m0 = 0; m0 < M; m0 += kMaxGridY * GM) {
        const int64_t rows = M - m0 < kMaxGridY * GM ? M - m0 : kMaxGridY * GM;
        dim3 grid(blocks_for(N, GN), blocks_for(rows, GM));
        hipLaunchKernelGGL(gemm_generic_kernel<true>, grid, dim3(256), 0, s, x + m0 * K, Wp, 1.f, scales, group,
                           y + m0 * N, rows, N, K, words);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_gemm3_generic(const __half* x, const uint8_t* Wp, int64_t stride, float gamma,
                                __half* y, int64_t M, int64_t N, int64_t K, bool fx, hipStream_t s)
{
    for (int64_t m0 = 0; m0 < M; m0 += kMaxGridY * MB) {
        const int64_t rows = M - m0 < kMaxGridY * MB ? M - m0 : kMaxGridY * MB;
        dim3 grid(blocks_for(N, 4), blocks_for(rows, MB));
        hipLaunchKernelGGL(gemm3_generic_kernel, grid, dim3(256), 0, s, x + m0 * K, Wp, stride, gamma, y + m0 * N, rows, N, K, fx);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace tl
