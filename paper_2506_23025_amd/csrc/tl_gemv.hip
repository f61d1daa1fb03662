// Weight-streaming small-M kernel for the 2-bit format (decode batches, M <= 16 per pass).
//
// The result it computes is App. B "Inference" of the paper, Y = X (gamma What)^T, with the
// Sec. 3.1 decode d = ((b >> 2j) & 3) - 1 done in registers.  How it is organised is ours:
//
//  * One workgroup owns a set of 16-row tiles of W; wave w of the group owns the K-slice
//    [512 (w + NW p), 512 (w + NW p) + 512) in pass p.  A wave therefore keeps its part of
//    the activations in registers (64 VGPRs per pass, laid out as MFMA B operands) and only
//    the packed weights stream: every byte of W is read exactly once, in full 128-byte
//    lines (8 adjacent lanes x dwordx4), non-temporally.
//  * The contraction runs on v_mfma_f32_16x16x32_f16 with W as the 16-row operand and the
//    (at most 16) activation rows as the 16 columns, so the cost per weight does not grow
//    with M.  Coalesced loads give a lane 16 bytes of ONE row; the MFMA wants lane
//    (i, g) to hold row i.  The 2 KB tile slice is turned through wave-private LDS
//    (ds_write_b128 / ds_read_b128, XOR-swizzled, no barrier: a wave only reads what it
//    wrote itself).
//  * Decode costs 11 VALU operations per 16 weights.  `word & (3 << 2j | 3 << (2j+16))`
//    leaves two codes in the mantissa fields of an fp16 pair, i.e. the subnormal numbers
//    c * 4^j * 2^-24 (gfx950 MFMA does not flush fp16 subnormals).  The matrix core aligns
//    products by their exponent FIELDS, so a code low in the mantissa loses accuracy
//    (measured: ~2^-17 relative at j = 0, none at j >= 3).  Three shifted copies of the
//    word (<< 4, >> 2, >> 8) therefore bring every code to j in {2, 3, 4}.  Products of
//    different j carry different power-of-two factors, so they go to three accumulators
//    that are combined once per tile: sum_j 2^(24-2j) acc_j = sum_k x_k c_k.  With
//    c = w + 1 the result is sum_k x_k c_k - sum_k x_k; the second sum is formed once per
//    wave from the activation registers.
//  * Split-K partial tiles of the NW waves are added in a fixed order through LDS, scaled
//    by gamma, rounded to fp16 (RNE) and stored.  No atomics: results are deterministic.
#include "tl_internal.hpp"

namespace tl {

namespace {

constexpr int kTMax = 8;          // tiles a workgroup keeps in flight
constexpr int kSliceK = 512;      // K elements a wave owns per pass
constexpr int kWaveLds = 16384;   // bytes of LDS per wave: 16 activation rows x 1 KB

struct GemvParams {
    const __half* x;
    const uint32_t* W;
    __half* y;
    float gamma;
    int M, N, K;
    int tiles;      // ceil(N / 16)
    int groups;     // gridDim.x
    int T;          // tiles per workgroup (<= kTMax)
    int slices;     // ceil(K / 512)
    int passes;     // ceil(slices / NW)
};

__device__ __forceinline__ u32x4 ldg_nt(const uint32_t* p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}

__device__ __forceinline__ f16x8 as_f16x8(u32x4 v)
{
    return __builtin_bit_cast(f16x8, v);
}

template <int TMAX>
__global__ void __launch_bounds__(512)
gemv_kernel(GemvParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int NW = blockDim.x >> 6;
    unsigned char* const my_lds = lds_raw + wave * kWaveLds;

    const int m0 = blockIdx.y * 16;
    const int Mrem = (p.M - m0 < 16) ? (p.M - m0) : 16;
    const int K = p.K;
    const int row_words = K >> 4;
    const int chunks = K >> 6;                 // 64-weight (16-byte) chunks per row

    // ---- coalesced load mapping: 8 lanes per 128-byte line, 8 rows per instruction ----
    const int lr = lane >> 3;                  // row within the half tile
    const int lc = lane & 7;                   // chunk within the slice
    // ---- MFMA mapping: lane (i, g) = (row / activation column, k group) -----------------
    const int mi = lane & 15;
    const int mg = lane >> 4;

    u32x4 wreg[TMAX][2];

    auto issue_w = [&](int t, int slice, u32x4 (&dst)[2]) {
        int tile = blockIdx.x + t * p.groups;
        if (tile >= p.tiles) tile = p.tiles - 1;          // duplicate work, never stored
        int chunk = slice * 8 + lc;
        if (chunk >= chunks) chunk = 0;                    // multiplied by zero activations
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            int row = tile * 16 + q * 8 + lr;
            if (row >= p.N) row = p.N - 1;
            dst[q] = ldg_nt(p.W + size_t(row) * row_words + chunk * 4);
        }
    };

    f32x4 part[TMAX];
#pragma unroll
    for (int t = 0; t < TMAX; ++t) part[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    float sx = 0.f;

    int slice = wave;
    if (slice < p.slices) {
#pragma unroll
        for (int t = 0; t < TMAX; ++t)
            if (t < p.T) issue_w(t, slice, wreg[t]);
    }

    for (int pass = 0; pass < p.passes; ++pass, slice += NW) {
        if (slice >= p.slices) break;                      // wave-uniform
        // ---------------- activations of this slice -> MFMA B registers ----------------
        // coalesced: one instruction per activation row, lane l takes 8 halves (16 bytes)
        u32x4 xraw[16];
        const int kx = slice * kSliceK + lane * 8;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            xraw[r] = u32x4{0u, 0u, 0u, 0u};
            if (r < Mrem && kx < K)
                xraw[r] = *reinterpret_cast<const u32x4*>(p.x + size_t(m0 + r) * K + kx);
        }
        // swizzled staging: row r, 16-byte piece (lane ^ (r & 7))
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (r < Mrem)
                *reinterpret_cast<u32x4*>(my_lds + r * 1024 + ((lane ^ (r & 7)) << 4)) = xraw[r];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // breg[h][wd][e]: (x[k], x[k + 8]) with k = slice0 + 64 (4h + g) + 16 wd + e
        uint32_t breg[2][4][8];
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int wd = 0; wd < 4; ++wd) {
                u32x4 lo = u32x4{0u, 0u, 0u, 0u}, hi = u32x4{0u, 0u, 0u, 0u};
                if (mi < Mrem) {
                    const int piece = 32 * h + 8 * mg + 2 * wd;     // 16-byte pieces of the row
                    lo = *reinterpret_cast<const u32x4*>(my_lds + mi * 1024 + (((piece) ^ (mi & 7)) << 4));
                    hi = *reinterpret_cast<const u32x4*>(my_lds + mi * 1024 + (((piece + 1) ^ (mi & 7)) << 4));
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    breg[h][wd][2 * r] = __builtin_amdgcn_perm(hi[r], lo[r], 0x05040100u);
                    breg[h][wd][2 * r + 1] = __builtin_amdgcn_perm(hi[r], lo[r], 0x07060302u);
                }
            }
        // sum of this lane's activations (each k of the slice sits in exactly one register half)
        {
            const f16x2 ones = {(_Float16)1.0f, (_Float16)1.0f};
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int wd = 0; wd < 4; ++wd)
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        sx = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, breg[h][wd][e]), ones, sx, false);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();

        // ---------------- stream the tiles of this slice ---------------------------------
        const bool more = (slice + NW) < p.slices;
#pragma unroll
        for (int t = 0; t < TMAX; ++t) {
            if (t < p.T) {
                unsigned char* tl_lds = my_lds + t * 2048;
                // turn the tile slice: [row][chunk ^ (row & 7)]
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int row = q * 8 + lr;
                    *reinterpret_cast<u32x4*>(tl_lds + row * 128 + ((lc ^ (row & 7)) << 4)) = wreg[t][q];
                }
                if (more) issue_w(t, slice + NW, wreg[t]);          // prefetch the next pass
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

                f32x4 acc[3];
#pragma unroll
                for (int j = 0; j < 3; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int cc = 4 * h + mg;
                    const u32x4 wv = *reinterpret_cast<const u32x4*>(tl_lds + mi * 128 + ((cc ^ (mi & 7)) << 4));
                    // element e of each half-word is moved to mantissa bits 4..9 (position
                    // class 2, 3 or 4): e = 0..2 by << 4, e = 3..5 by >> 2, e = 6..7 by >> 8
                    const u32x4 sh[3] = {wv << 4, wv >> 2, wv >> 8};
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int j = e % 3;                        // accumulator: class j + 2
                        const uint32_t mask = 0x00300030u << (2 * j);
                        const u32x4 a = sh[e / 3] & mask;
                        const u32x4 b = u32x4{breg[h][0][e], breg[h][1][e], breg[h][2][e], breg[h][3][e]};
                        acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(a), as_f16x8(b), acc[j], 0, 0, 0);
                    }
                }
                // fp16 bits c << (2j + 4) are the subnormal c 4^(j+2) 2^-24: undo with 2^(20 - 2j)
                part[t] += acc[0] * 1048576.f + acc[1] * 262144.f + acc[2] * 65536.f;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }

    // ---- sum_k x_k over the wave's slices, for this lane's activation column -----------
    sx += __shfl_xor(sx, 16, 64);
    sx += __shfl_xor(sx, 32, 64);

    // ---- split-K reduction across the waves, epilogue -----------------------------------
    // Layout [t][wave][lane] of f32x4 in LDS (reuses the staging space after a barrier).
    __syncthreads();
    f32x4* red = reinterpret_cast<f32x4*>(lds_raw);
#pragma unroll
    for (int t = 0; t < TMAX; ++t)
        if (t < p.T) red[(t * NW + wave) * 64 + lane] = part[t] - sx;
    __syncthreads();
    for (int item = threadIdx.x; item < p.T * 64; item += blockDim.x) {
        const int t = item >> 6;
        const int l = item & 63;
        const int tile = blockIdx.x + t * p.groups;
        if (tile >= p.tiles) continue;
        f32x4 s = red[(t * NW) * 64 + l];
        for (int w = 1; w < NW; ++w) s += red[(t * NW + w) * 64 + l];
        const int m = m0 + (l & 15);
        const int n = tile * 16 + 4 * (l >> 4);
        if ((l & 15) < Mrem) {
            __half* dst = p.y + size_t(m) * p.N + n;
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (n + r < p.N) dst[r] = __float2half_rn(p.gamma * s[r]);
        }
    }
}

}  // namespace

bool gemv_supports(int64_t M, int64_t N, int64_t K)
{
    return M >= 1 && N >= 1 && K >= 64 && (K % 64) == 0 && K <= (int64_t(1) << 24) &&
           N <= (int64_t(1) << 24) && (M + 15) / 16 <= 65535;
}

hipError_t launch_gemv(const __half* x, const uint32_t* Wp, float gamma, __half* y,
                       int64_t M, int64_t N, int64_t K, hipStream_t s)
{
    GemvParams p;
    p.x = x; p.W = Wp; p.y = y; p.gamma = gamma;
    p.M = int(M); p.N = int(N); p.K = int(K);
    p.tiles = int((N + 15) / 16);
    p.slices = int((K + kSliceK - 1) / kSliceK);
    const int NW = p.slices < 8 ? p.slices : 8;
    p.passes = (p.slices + NW - 1) / NW;
    int groups = p.tiles < 256 ? p.tiles : 256;
    int T = (p.tiles + groups - 1) / groups;
    if (T > kTMax) { T = kTMax; groups = (p.tiles + T - 1) / T; }
    p.groups = groups; p.T = T;
    const size_t lds = size_t(NW) * kWaveLds;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemv_kernel<kTMax>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 8 * kWaveLds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid(groups, unsigned((M + 15) / 16));
    hipLaunchKernelGGL(gemv_kernel<kTMax>, grid, dim3(NW * 64), lds, s, p);
    return hipGetLastError();
}

}  // namespace tl
