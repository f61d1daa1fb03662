// Weight-streaming small-M kernel for the 1.6-bit format (5 trits per byte, plain base 3:
// byte = sum_i (w_i + 1) 3^i, the block code of Sec. 3.2 without its fixed-point scaling).
//
// Same organisation as the 2-bit kernel (tl_gemv.hip): a workgroup owns 16-row tiles, wave w
// owns a K slice and keeps its activations in registers as MFMA B operands, packed rows
// stream once in full 128-byte lines, the tile slice is turned into MFMA order through
// wave-private LDS, split-K partial tiles are summed through LDS in a fixed order.
// What differs is the slice geometry and the decode:
//
//  * A slice is 128 packed bytes = 640 weights per row; a lane's 16 bytes hold 80 weights.
//  * Decode is a table look-up: a 256-entry table of 8-byte entries in LDS maps a byte to its
//    five digits c = w + 1 as fp16 (subnormal) pairs: word 0 = c0 << 6 | c2 << 8 | c3 << 22,
//    word 1 = c1 << 6 | c4 << 22 (every digit at bit 6 or above of its half: the matrix
//    instruction aligns products by exponent field, and subnormals with only their lowest bits set
//    lose low-order product bits).  The two words of two neighbouring bytes, with c2 masked out
//    of the first word of each, are one A operand of v_mfma_f32_16x16x32_f16 as they stand:
//    (c0, c3) 2^-18, (c1, c4) 2^-18 per byte, against the activation pairs (x[5b], x[5b+3]) and
//    (x[5b+1], x[5b+4]); the c2 digits of four bytes, masked out the other way, are a third
//    operand (c2, 0) 2^-16 against (x[5b+2], 0).  Per 5 weights: 1 address operation (a shift
//    with a byte select), 1 LDS read, 2 ANDs; all sixteen look-ups of a half tile are issued
//    before the first is used.
//  * The paper expects the 1.6-bit form to cost more arithmetic per weight than the 2-bit
//    form (Sec. 3.3 results, "Limitations"); here it is 0.7 VALU operations and 0.2 LDS
//    look-ups per weight against 0.7 VALU operations for the 2-bit form, for 0.81 of the
//    bytes, and 24 MFMAs per 640 x 16 weights against 16 per 512 x 16: per weight the SIMD time
//    is the same, per byte of packed weights it is 1.25 times the 2-bit kernel's.
//  * Two forms.  gemv3_stream_kernel (K in one pass of at most 7 slices, K <= 4480): a wave
//    keeps its slice, a workgroup walks a run of tiles in items with the next item's weights in
//    flight; gemv3_grouped_kernel is the same body fed from one record per workgroup, so that
//    one launch carries several GEMMs.  gemv3_kernel (longer K): waves loop over slices, one
//    item per workgroup.
#include "tl_internal.hpp"
#include "tl_deal.hpp"

#include <type_traits>

namespace tl {

namespace {

constexpr int kT3Max = 4;            // tiles per workgroup
constexpr int kSlice3 = 640;         // weights per slice (128 packed bytes)
constexpr int kXRow = 1296;          // bytes per staged activation row (1280 + 16: spreads LDS banks)
constexpr int kWave3Lds = 16 * kXRow;   // 20736 bytes per wave
constexpr int kLutBytes = 2048;       // 256 entries of 8 bytes
constexpr int kNW3Max = 7;           // 7 * 20736 + 2048 bytes of LDS

struct Gemv3Params {
    const __half* x;
    const uint8_t* W;
    __half* y;
    float gamma;
    int M, N, K;
    int stride;      // bytes per packed row (multiple of 16)
    int tiles;       // ceil(N / 16)
    int groups;      // gridDim.x
    int slices;      // ceil(stride / 128)
    int fx;          // bytes hold the fixed-point code of Sec. 3.2 instead of plain base 3
};

constexpr int vmcnt_imm3(int n)
{
    return (n & 0xF) | ((n >> 4) << 14) | (0x7 << 4) | (0xF << 8);
}

__device__ __forceinline__ f16x8 as_h8(u32x4 v) { return __builtin_bit_cast(f16x8, v); }

// Barrier that waits for this wave's LDS traffic only; the weight loads and activation
// transfers already requested stay in flight across it (__syncthreads would drain them).
__device__ __forceinline__ void lds_barrier3()
{
    __builtin_amdgcn_s_waitcnt(0xF | (0x3 << 14) | (0x7 << 4));      // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
}

// 8 * (byte B of w): the offset of that byte's table entry, in one instruction (the shift
// reads its operand through a byte select).
template <int B>
__device__ __forceinline__ uint32_t byte_times_8(uint32_t w)
{
    uint32_t r;
    const uint32_t three = 3u;
    if constexpr (B == 0) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0" : "=v"(r) : "v"(three), "v"(w));
    if constexpr (B == 1) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(r) : "v"(three), "v"(w));
    if constexpr (B == 2) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2" : "=v"(r) : "v"(three), "v"(w));
    if constexpr (B == 3) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(r) : "v"(three), "v"(w));
    return r;
}

// byte -> digits table.  Plain form: base-3 digits, least significant first (bytes 243..255
// never occur; they decode like byte - 243).  Fixed-point form (Sec. 3.2): the block value is
// floor(243 b / 256), the inverse of b = ceil(256 V / 243), and its base-3 digits go most
// significant first; all 256 bytes decode, and to the digits App. F, Alg. 1 gives.
__device__ __forceinline__ void fill_table(u32x2* lut, bool fx)
{
    for (unsigned b = threadIdx.x; b < 256; b += blockDim.x) {
        unsigned c[5];
        if (fx) {
            unsigned v = (b * 243u) >> 8;
#pragma unroll
            for (int i = 4; i >= 0; --i) { c[i] = v % 3u; v /= 3u; }
        } else {
            unsigned v = b >= 243 ? b - 243 : b;
#pragma unroll
            for (int i = 0; i < 5; ++i) { c[i] = v % 3u; v /= 3u; }
        }
        lut[b] = u32x2{(c[0] << 6) | (c[2] << 8) | (c[3] << 22), (c[1] << 6) | (c[4] << 22)};
    }
}

// The activations as MFMA B operands, grouped as the tile arithmetic uses them.  With
// p(a, b) = (x[a], x[b]) and k = 5 (4d + j) the first weight of byte 4d + j of the lane's 16 bytes of
// half h:  bop[h][d][0] = p(k0, k0+3), p(k0+1, k0+4) for bytes j = 0, 1;  bop[h][d][1] the same for
// j = 2, 3;  bop[h][d][2] = (x[k+2], 0) for j = 0..3.  The lane's 16 bytes of half h cover 80
// consecutive weights, i.e. 160 consecutive bytes of the staged row: ten 16-byte reads, then one
// byte permute per pair.
__device__ __forceinline__ void build_operands(const unsigned char* row, int mg, u32x4 (&bop)[2][4][3])
{
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        u32x4 xv[10];
#pragma unroll
        for (int i = 0; i < 10; ++i)
            xv[i] = *reinterpret_cast<const u32x4*>(row + (4 * h + mg) * 160 + 16 * i);
        auto pair = [&](int a, int b) {                    // (x[a], x[b]) of the 80; b < 0: (x[a], 0)
            const uint32_t lo = xv[a >> 3][(a >> 1) & 3];
            const uint32_t hi = b < 0 ? 0u : xv[b >> 3][(b >> 1) & 3];
            const uint32_t s0 = (a & 1) ? 0x0302u : 0x0100u;
            const uint32_t s1 = b < 0 ? 0x0c0cu : ((b & 1) ? 0x0706u : 0x0504u);
            return __builtin_amdgcn_perm(hi, lo, (s1 << 16) | s0);
        };
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int k = 20 * d;                           // first weight of byte 4d
            bop[h][d][0] = u32x4{pair(k, k + 3), pair(k + 1, k + 4), pair(k + 5, k + 8), pair(k + 6, k + 9)};
            bop[h][d][1] = u32x4{pair(k + 10, k + 13), pair(k + 11, k + 14), pair(k + 15, k + 18), pair(k + 16, k + 19)};
            bop[h][d][2] = u32x4{pair(k + 2, -1), pair(k + 7, -1), pair(k + 12, -1), pair(k + 17, -1)};
        }
    }
}

// -2^-18 sum_k x over the slice, in accumulator layout (constant 16-row operand)
__device__ __forceinline__ f32x4 seed_from(const u32x4 (&bop)[2][4][3])
{
    f32x4 nsx = f32x4{0.f, 0.f, 0.f, 0.f};
    const uint32_t c = 0x80408040u;
    const u32x4 a = u32x4{c, c, c, c};
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
            for (int q = 0; q < 3; ++q)
                nsx = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(a), as_h8(bop[h][d][q]), nsx, 0, 0, 0);
    return nsx;
}

// sum_k x_k w_k of one tile slice that lies in MFMA order at reg_t: all sixteen look-ups of a
// half first, so that their latency runs under the arithmetic of the ones before
template <class LutAt>
__device__ __forceinline__ f32x4 tile_sum(const unsigned char* reg_t, uint32_t wr_off0, uint32_t wr_off1,
                                          const u32x4 (&bop)[2][4][3], f32x4 nsx, LutAt lut_at)
{
    f32x4 acc[3] = {nsx, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const u32x4 wv = *reinterpret_cast<const u32x4*>(reg_t + (h ? wr_off1 : wr_off0));
        u32x2 e[4][4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            e[d][0] = lut_at(byte_times_8<0>(wv[d]));
            e[d][1] = lut_at(byte_times_8<1>(wv[d]));
            e[d][2] = lut_at(byte_times_8<2>(wv[d]));
            e[d][3] = lut_at(byte_times_8<3>(wv[d]));
        }
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            // bytes 0,1 and 2,3 of the dword: the two table words of a byte pair are an operand
            // as they stand once c2 is masked out of the first word of each
            const u32x4 a2 = u32x4{e[d][0][0] & 0x300u, e[d][1][0] & 0x300u, e[d][2][0] & 0x300u, e[d][3][0] & 0x300u};
            const u32x4 a01 = u32x4{e[d][0][0] & 0x00c000c0u, e[d][0][1], e[d][1][0] & 0x00c000c0u, e[d][1][1]};
            const u32x4 a23 = u32x4{e[d][2][0] & 0x00c000c0u, e[d][2][1], e[d][3][0] & 0x00c000c0u, e[d][3][1]};
            acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(a01), as_h8(bop[h][d][0]), acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(a23), as_h8(bop[h][d][1]), acc[1], 0, 0, 0);
            acc[2] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(a2), as_h8(bop[h][d][2]), acc[2], 0, 0, 0);
        }
    }
    return (acc[0] + acc[1]) * 262144.f + acc[2] * 65536.f;
}

template <int T>
__global__ void __launch_bounds__(512)
gemv3_kernel(Gemv3Params p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int NW = blockDim.x >> 6;
    u32x2* const lut = reinterpret_cast<u32x2*>(lds_raw);
    unsigned char* const my_lds = lds_raw + kLutBytes + wave * kWave3Lds;
    // the table starts the LDS: a byte offset into it is an LDS address
    auto lut_at = [](uint32_t off) { return *(const __attribute__((address_space(3))) u32x2*)(uintptr_t(off)); };

    const int m0 = blockIdx.y * 16;
    const int Mrem = (p.M - m0 < 16) ? (p.M - m0) : 16;
    int MR = 1;
    while (MR < Mrem) MR *= 2;
    const int K = p.K, N = p.N;
    const uint32_t stride = uint32_t(p.stride);
    const int chunks = p.stride >> 4;          // 16-byte chunks per packed row
    const int grp = blockIdx.x, groups = p.groups, tiles = p.tiles, slices = p.slices;

    const int lr = lane >> 3, lc = lane & 7;   // load mapping: row of the half tile, chunk of the slice
    const int mi = lane & 15, mg = lane >> 4;  // MFMA mapping: row / activation column, k group
    const int xrow = mi & (MR - 1);

    const uint32_t ww_off = uint32_t(lr) * 128u + (uint32_t(lc ^ lr) << 4);
    const uint32_t wr_off0 = uint32_t(mi) * 128u + (uint32_t((mg) ^ (mi & 7)) << 4);
    const uint32_t wr_off1 = uint32_t(mi) * 128u + (uint32_t((4 + mg) ^ (mi & 7)) << 4);

    const unsigned char* const Wb = p.W;
    const unsigned char* const xb = reinterpret_cast<const unsigned char*>(p.x + size_t(m0) * K);

    u32x4 wreg[T][2];
    const bool ragged_n = (N & 15) != 0;
    auto issue_w = [&](int t, int slice) {
        int tile = grp + t * groups;
        if (tile >= tiles) tile = tiles - 1;
        int chunk = slice * 8 + lc;
        if (chunk >= chunks) chunk = 0;                    // past the row: meets zero activations
        const unsigned char* tb = Wb + size_t(tile) * 16u * stride;
        uint32_t off0 = uint32_t(lr) * stride + uint32_t(chunk) * 16u;
        uint32_t off1 = off0 + 8u * stride;
        if (ragged_n && tile == tiles - 1) {
            const int last = N - 1 - tile * 16;
            off0 = uint32_t(lr < last ? lr : last) * stride + uint32_t(chunk) * 16u;
            off1 = uint32_t(lr + 8 < last ? lr + 8 : last) * stride + uint32_t(chunk) * 16u;
        }
        wreg[t][0] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tb + off0));
        wreg[t][1] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tb + off1));
    };

    // Staged activation row r of the slice: 640 halves = 80 pieces of 16 bytes, by LDS-DMA
    // (two instructions: pieces 0..63, then 64..79).  Pieces past K are stored as zeros.
    auto issue_x = [&](int slice) {
        // rows past Mrem stay unwritten: an MFMA column depends on its own column of B alone,
        // and the outputs of those columns are not stored
        for (int r = 0; r < Mrem; ++r) {
            const unsigned char* src = xb + size_t(r) * K * 2;
            unsigned char* dst = my_lds + r * kXRow;
#pragma unroll
            for (int part = 0; part < 2; ++part) {
                const int piece = part * 64 + lane;
                const int kx = slice * kSlice3 + piece * 8;
                if (piece < 80) {
                    if (kx < K) {
                        __builtin_amdgcn_global_load_lds(
                            (const __attribute__((address_space(1))) void*)(src + uint32_t(kx) * 2u),
                            (__attribute__((address_space(3))) void*)(dst + part * 1024),
                            16, 0, 0);
                    } else {
                        *reinterpret_cast<u32x4*>(dst + piece * 16) = u32x4{0u, 0u, 0u, 0u};
                    }
                }
            }
        }
    };

    f32x4 part_acc[T];
#pragma unroll
    for (int t = 0; t < T; ++t) part_acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    int slice = wave;
    if (slice < slices) {
        issue_x(slice);
#pragma unroll
        for (int t = 0; t < T; ++t) issue_w(t, slice);
    }

    fill_table(lut, p.fx != 0);
    // (the barrier that makes the table visible comes after the operands are built: they need
    // the wave's own activation transfers only)
    if (wave < slices) __builtin_amdgcn_s_waitcnt(vmcnt_imm3(2 * T));   // LDS-DMA is not tracked by the compiler

    for (; slice < slices; slice += NW) {
        const bool more = (slice + NW) < slices;
        u32x4 bop[2][4][3];
        build_operands(my_lds + xrow * kXRow, mg, bop);
        const f32x4 nsx = seed_from(bop);
        if (slice == wave) lds_barrier3();                 // first pass (every wave runs it): the table is complete
#pragma unroll
        for (int t = 0; t < T; ++t) {
            unsigned char* const reg_t = my_lds + t * 2048;
            *reinterpret_cast<u32x4*>(reg_t + ww_off) = wreg[t][0];
            *reinterpret_cast<u32x4*>(reg_t + 1024 + ww_off) = wreg[t][1];
            if (more) issue_w(t, slice + NW);
            if (grp + t * groups < tiles) part_acc[t] += tile_sum(reg_t, wr_off0, wr_off1, bop, nsx, lut_at);
        }
        if (more) {
            issue_x(slice + NW);
            __builtin_amdgcn_s_waitcnt(vmcnt_imm3(0));
        }
    }

    // ---- split-K reduction across the waves, epilogue ----
    lds_barrier3();
    f32x4* red = reinterpret_cast<f32x4*>(lds_raw + kLutBytes);
#pragma unroll
    for (int t = 0; t < T; ++t) red[(t * NW + wave) * 64 + lane] = part_acc[t];
    lds_barrier3();
    for (int item = threadIdx.x; item < T * 64; item += blockDim.x) {
        const int t = item >> 6;
        const int l = item & 63;
        const int tile = grp + t * groups;
        if (tile >= tiles) continue;
        f32x4 v[8];
#pragma unroll
        for (int w = 0; w < 8; ++w)
            v[w] = (w < NW) ? red[(t * NW + w) * 64 + l] : f32x4{0.f, 0.f, 0.f, 0.f};
        const f32x4 s = ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
        const int n = tile * 16 + 4 * (l >> 4);
        if ((l & 15) < Mrem) {
            __half* dst = p.y + size_t(m0 + (l & 15)) * N + n;
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (n + r < N) dst[r] = __float2half_rn(p.gamma * s[r]);
        }
    }
}

// ------------------------------------------------------------------------------------------
// Stream form, for K of at most 7 slices (K <= 4480): wave w owns slice w for the whole kernel,
// so activations are staged and turned into operands once; a workgroup walks a run of
// consecutive tiles, T at a time ("item"), with the next item's weights requested as soon as
// a tile's registers are free, two alternating sets of partial sums and one LDS-only barrier
// per item -- the organisation of the 2-bit stream kernel (tl_gemv.hip) with this file's
// decode.  Params::groups workgroups; workgroup g takes tiles [g per + min(g, extra), ...).
// What a workgroup of the stream form works on: one block of at most 16 activation rows of one
// GEMM and a run of consecutive tiles of its matrix.  x and y point at the block's first row.
struct Run3 {
    const unsigned char* W;   // the matrix (first row)
    const unsigned char* x;
    __half* y;
    float gamma;
    int K, N;
    int stride;               // bytes per packed row
    int Mrem;                 // activation rows, 1..16
    int tile0, tile_end;      // the run
    int slices;               // waves with a slice of K (the others idle along)
    int fx;                   // which byte code the table is filled for
};
static_assert(sizeof(Run3) == 64, "one record per 64-byte line");

constexpr int kRec3Max = 256;  // records (workgroups) of a grouped launch: 16 KB of kernel arguments

struct Rec3Batch {
    Run3 rec[kRec3Max];
};

template <int T>
__device__ __forceinline__ void gemv3_stream_body(const Run3& p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int NW = blockDim.x >> 6;
    u32x2* const lut = reinterpret_cast<u32x2*>(lds_raw);
    unsigned char* const my_lds = lds_raw + kLutBytes + wave * kWave3Lds;
    auto lut_at = [](uint32_t off) { return *(const __attribute__((address_space(3))) u32x2*)(uintptr_t(off)); };

    const int Mrem = p.Mrem;
    int MR = 1;
    while (MR < Mrem) MR *= 2;
    const int K = p.K, N = p.N;
    const uint32_t stride = uint32_t(p.stride);
    const int chunks = p.stride >> 4;
    const int tiles = (N + 15) >> 4;
    const int tile0 = p.tile0;
    const int tile_end = p.tile_end;
    const int n_items = (tile_end - tile0 + T - 1) / T;

    const int lr = lane >> 3, lc = lane & 7;
    const int mi = lane & 15, mg = lane >> 4;
    const int xrow = mi & (MR - 1);
    const uint32_t ww_off = uint32_t(lr) * 128u + (uint32_t(lc ^ lr) << 4);
    const uint32_t wr_off0 = uint32_t(mi) * 128u + (uint32_t((mg) ^ (mi & 7)) << 4);
    const uint32_t wr_off1 = uint32_t(mi) * 128u + (uint32_t((4 + mg) ^ (mi & 7)) << 4);

    const unsigned char* const Wb = p.W;
    const unsigned char* const xb = p.x;
    const bool active = wave < p.slices;
    uint32_t col_off;
    {
        int chunk = wave * 8 + lc;
        if (chunk >= chunks) chunk = 0;                    // past the row: meets zero activations
        col_off = uint32_t(chunk) * 16u;
    }
    const bool ragged_n = (N & 15) != 0;
    typedef const __attribute__((address_space(1))) u32x4* gptr;

    u32x4 wreg[T][2];
    auto issue_w = [&](int first, int t) {
        int tile = first + t;
        if (tile >= tile_end) tile = tile_end - 1;         // past the run: its last tile again, never stored
        const unsigned char* tb = Wb + size_t(tile) * 16u * stride;
        const int last = (ragged_n && tile == tiles - 1) ? N - 1 - tile * 16 : 15;
        const uint32_t off0 = uint32_t(lr < last ? lr : last) * stride + col_off;
        const uint32_t off1 = uint32_t(lr + 8 < last ? lr + 8 : last) * stride + col_off;
        wreg[t][0] = __builtin_nontemporal_load((gptr)(tb + off0));
        wreg[t][1] = __builtin_nontemporal_load((gptr)(tb + off1));
    };

    if (active) {
        // activation rows of this wave's slice by LDS-DMA: 640 halves = 80 pieces of 16 bytes per
        // row (pieces 0..63, then 64..79); pieces past K are stored as zeros; rows past Mrem stay
        // unwritten (an MFMA column depends on its own column of B alone)
        for (int r = 0; r < Mrem; ++r) {
            const unsigned char* src = xb + size_t(r) * K * 2;
            unsigned char* dst = my_lds + r * kXRow;
#pragma unroll
            for (int part = 0; part < 2; ++part) {
                const int piece = part * 64 + lane;
                const int kx = wave * kSlice3 + piece * 8;
                if (piece < 80) {
                    if (kx < K) {
                        __builtin_amdgcn_global_load_lds(
                            (const __attribute__((address_space(1))) void*)(src + uint32_t(kx) * 2u),
                            (__attribute__((address_space(3))) void*)(dst + part * 1024), 16, 0, 0);
                    } else {
                        *reinterpret_cast<u32x4*>(dst + piece * 16) = u32x4{0u, 0u, 0u, 0u};
                    }
                }
            }
        }
#pragma unroll
        for (int t = 0; t < T; ++t) issue_w(tile0, t);
    }
    fill_table(lut, p.fx != 0);
    if (active) __builtin_amdgcn_s_waitcnt(vmcnt_imm3(2 * T));   // the activations are in; the weights stay in flight

    u32x4 bop[2][4][3];
    f32x4 nsx = f32x4{0.f, 0.f, 0.f, 0.f};
    if (active) {
        build_operands(my_lds + xrow * kXRow, mg, bop);
        nsx = seed_from(bop);
    }
    lds_barrier3();                                        // the table is complete

    auto item = [&](auto refill_tag, int first, int parity) {
        constexpr bool REFILL = decltype(refill_tag)::value;
        f32x4 part[T];
#pragma unroll
        for (int t = 0; t < T; ++t) part[t] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (active) {
#pragma unroll
            for (int t = 0; t < T; ++t) {
                unsigned char* const reg_t = my_lds + (t & 1) * 2048;
                *reinterpret_cast<u32x4*>(reg_t + ww_off) = wreg[t][0];
                *reinterpret_cast<u32x4*>(reg_t + 1024 + ww_off) = wreg[t][1];
                if constexpr (REFILL) issue_w(first + T, t);
                if (REFILL || first + t < tile_end)
                    part[t] = tile_sum(reg_t, wr_off0, wr_off1, bop, nsx, lut_at);
            }
        }
        unsigned char* const red = my_lds + 4096 + parity * (T * 1024);
#pragma unroll
        for (int t = 0; t < T; ++t) reinterpret_cast<f32x4*>(red + t * 1024)[lane] = part[t];
        lds_barrier3();
        if (const int o = threadIdx.x; o < T * 64) {       // T <= waves: one output quad per thread
            const int t = o >> 6, l = o & 63;
            const int tile = first + t;
            f32x4 v[8];
#pragma unroll
            for (int w = 0; w < 8; ++w)
                v[w] = (w < NW) ? reinterpret_cast<const f32x4*>(lds_raw + kLutBytes + w * kWave3Lds + 4096 + parity * (T * 1024) + t * 1024)[l]
                                : f32x4{0.f, 0.f, 0.f, 0.f};
            const f32x4 s = ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
            const int n = tile * 16 + 4 * (l >> 4);
            if (tile < tile_end && (l & 15) < Mrem) {
                typedef __attribute__((address_space(1))) __half* gh_ptr;
                gh_ptr dst = (gh_ptr)(p.y + size_t(l & 15) * N + n);
                const float gamma = p.gamma;
                if (n + 3 < N && (N & 3) == 0) {           // four consecutive n: one 8-byte store
                    const f16x2 lo = {(_Float16)(gamma * s[0]), (_Float16)(gamma * s[1])};
                    const f16x2 hi = {(_Float16)(gamma * s[2]), (_Float16)(gamma * s[3])};
                    *(__attribute__((address_space(1))) u32x2*)dst =
                        u32x2{__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (n + r < N) *(__attribute__((address_space(1))) _Float16*)(dst + r) = (_Float16)(gamma * s[r]);
                }
            }
        }
    };
    int i = 0;
    for (; i + 1 < n_items; ++i) item(std::true_type{}, tile0 + i * T, i & 1);
    item(std::false_type{}, tile0 + i * T, i & 1);
}

// One GEMM: blockIdx.y is the block of 16 activation rows, the tiles are split evenly over gridDim.x.
template <int T>
__global__ void __launch_bounds__(512)
gemv3_stream_kernel(Gemv3Params p)
{
    const int m0 = blockIdx.y * 16;
    const int per = p.tiles / p.groups, extra = p.tiles % p.groups;
    const int g = blockIdx.x;
    Run3 r;
    r.W = p.W;
    r.x = reinterpret_cast<const unsigned char*>(p.x + size_t(m0) * p.K);
    r.y = p.y + size_t(m0) * p.N;
    r.gamma = p.gamma;
    r.K = p.K; r.N = p.N; r.stride = p.stride;
    r.Mrem = (p.M - m0 < 16) ? (p.M - m0) : 16;
    r.tile0 = g * per + (g < extra ? g : extra);
    r.tile_end = r.tile0 + per + (g < extra ? 1 : 0);
    r.slices = p.slices;
    r.fx = p.fx;
    gemv3_stream_body<T>(r);
}

// Several GEMMs: the host has dealt out the workgroups and written one record for each.
template <int T>
__global__ void __launch_bounds__(512)
gemv3_grouped_kernel(Rec3Batch b)
{
    gemv3_stream_body<T>(b.rec[blockIdx.x]);
}

using Kernel3Fn = void (*)(Gemv3Params);

Kernel3Fn pick3(int T)
{
    switch (T) {
        case 1: return gemv3_kernel<1>;
        case 2: return gemv3_kernel<2>;
        case 3: return gemv3_kernel<3>;
        default: return gemv3_kernel<4>;
    }
}

Kernel3Fn pick3_stream(int T)
{
    switch (T) {
        case 1: return gemv3_stream_kernel<1>;
        case 2: return gemv3_stream_kernel<2>;
        default: return gemv3_stream_kernel<3>;
    }
}

using Grouped3Fn = void (*)(Rec3Batch);

Grouped3Fn pick3_grouped(int T)
{
    switch (T) {
        case 1: return gemv3_grouped_kernel<1>;
        case 2: return gemv3_grouped_kernel<2>;
        default: return gemv3_grouped_kernel<3>;
    }
}

constexpr int kMaxBlocks3 = 32;          // blocks of 16 activation rows per grouped launch

}  // namespace

hipError_t gemv3_init()
{
    for (int T = 1; T <= kT3Max; ++T) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(pick3(T)),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           kNW3Max * kWave3Lds + kLutBytes);
        if (e == hipSuccess && T <= 3)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(pick3_stream(T)),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kNW3Max * kWave3Lds + kLutBytes);
        if (e == hipSuccess && T <= 3)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(pick3_grouped(T)),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kNW3Max * kWave3Lds + kLutBytes);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

bool gemv3_supports(int64_t M, int64_t N, int64_t K)
{
    return M >= 1 && N >= 1 && K >= 8 && (K % 8) == 0 && K <= (int64_t(1) << 24) &&
           N <= (int64_t(1) << 24) && (M + 15) / 16 <= 65535;
}

bool gemv3_groups(int64_t M, int64_t N, int64_t K)
{
    // K in one pass of the stream form: at most kNW3Max slices of 128 packed bytes
    return gemv3_supports(M, N, K) && (K + 4) / 5 <= int64_t(kNW3Max) * 128;
}

// Several GEMMs in one launch of the stream form: every block of 16 activation rows of every GEMM
// is a job, the 256 workgroups are dealt out to the jobs (tl_deal.hpp; the cost model is the one
// measured for the 2-bit kernel, whose item structure this kernel shares), and each workgroup
// gets a record with its run.
hipError_t launch_gemv3_jobs(const Gemm3Desc* jobs, int count, bool fx, hipStream_t s)
{
    for (int i = 0; i < count; ++i)
        if (!gemv3_groups(jobs[i].M, jobs[i].N, jobs[i].K)) return hipErrorInvalidValue;
    struct Block { int job; int64_t m0; int rows; };
    Block blk[kMaxBlocks3];
    int nb = 0;
    static bool lds_raised[kMaxDevices][4];
    auto flush = [&]() -> hipError_t {
        if (nb == 0) return hipSuccess;
        DealJob dj[kMaxBlocks3];
        int NW = 1;
        int64_t total_tiles = 0;
        for (int q = 0; q < nb; ++q) {
            const Gemm3Desc& d = jobs[blk[q].job];
            const int tiles = int((d.N + 15) / 16);
            const int slices = int((d.stride + 127) / 128);
            dj[q] = DealJob{tiles, 1, 0.15 * double(blk[q].rows)};
            total_tiles += tiles;
            if (slices > NW) NW = slices;
        }
        const int G = total_tiles < kRec3Max ? int(total_tiles) : kRec3Max;
        const DealModel model{3, true, 2.1, 0.43};
        int wg[kMaxBlocks3];
        deal_workgroups(model, dj, nb, G, wg);
        int run = 1, grid = 0;
        for (int q = 0; q < nb; ++q) {
            const int r = (dj[q].tiles + wg[q] - 1) / wg[q];
            if (r > run) run = r;
            grid += wg[q];
        }
        if (grid > kRec3Max) return hipErrorInvalidValue;   // more jobs than workgroups: cannot happen with kMaxBlocks3 <= kRec3Max
        int T = run <= 3 ? run : (run == 4 ? 2 : 3);
        if (T > NW) T = NW;                                // the epilogue gives every thread at most one output quad
        Rec3Batch rb;
        int g = 0;
        for (int q = 0; q < nb; ++q) {
            const Gemm3Desc& d = jobs[blk[q].job];
            const int per = dj[q].tiles / wg[q], plus = dj[q].tiles % wg[q];
            for (int w = 0; w < wg[q]; ++w) {
                Run3& r = rb.rec[g++];
                r.W = d.W;
                r.x = reinterpret_cast<const unsigned char*>(d.x + blk[q].m0 * d.K);
                r.y = d.y + blk[q].m0 * d.N;
                r.gamma = d.gamma;
                r.K = int(d.K); r.N = int(d.N); r.stride = int(d.stride);
                r.Mrem = blk[q].rows;
                r.tile0 = w * per + (w < plus ? w : plus);
                r.tile_end = r.tile0 + per + (w < plus ? 1 : 0);
                r.slices = int((d.stride + 127) / 128);
                r.fx = fx ? 1 : 0;
            }
        }
        Grouped3Fn fn = pick3_grouped(T);
        const int dev = device_slot();
        if (dev < 0 || !lds_raised[dev][T]) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize,
                                                     kNW3Max * kWave3Lds + kLutBytes);
            if (e != hipSuccess) return e;
            if (dev >= 0) lds_raised[dev][T] = true;
        }
        hipLaunchKernelGGL(fn, dim3(grid), dim3(NW * 64), size_t(NW) * kWave3Lds + kLutBytes, s, rb);
        nb = 0;
        return hipGetLastError();
    };
    for (int i = 0; i < count; ++i) {
        for (int64_t m0 = 0; m0 < jobs[i].M; m0 += 16) {
            blk[nb++] = Block{i, m0, int(jobs[i].M - m0 < 16 ? jobs[i].M - m0 : 16)};
            if (nb == kMaxBlocks3) {
                const hipError_t e = flush();
                if (e != hipSuccess) return e;
            }
        }
    }
    return flush();
}

hipError_t launch_gemv3(const __half* x, const uint8_t* Wp, int64_t stride, float gamma, __half* y,
                        int64_t M, int64_t N, int64_t K, bool fx, hipStream_t s)
{
    Gemv3Params p;
    p.fx = fx ? 1 : 0;
    p.x = x; p.W = Wp; p.y = y; p.gamma = gamma;
    p.M = int(M); p.N = int(N); p.K = int(K);
    p.stride = int(stride);
    p.tiles = int((N + 15) / 16);
    p.slices = int((stride + 127) / 128);
    const int NW = p.slices < kNW3Max ? p.slices : kNW3Max;
    int groups = p.tiles < 256 ? p.tiles : 256;
    static bool lds_raised[kMaxDevices][2][kT3Max + 1];
    const int dev = device_slot();
    auto raise = [&](Kernel3Fn fn, int form, int T) -> hipError_t {
        if (dev >= 0 && lds_raised[dev][form][T]) return hipSuccess;
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize,
                                                 kNW3Max * kWave3Lds + kLutBytes);
        if (e == hipSuccess && dev >= 0) lds_raised[dev][form][T] = true;
        return e;
    };
    dim3 grid(groups, unsigned((M + 15) / 16));
    if (p.slices <= kNW3Max) {
        // every block of 16 activation rows is a set of workgroups of its own (blockIdx.y); they
        // share the CUs, 256 workgroups in all, so that the launch is one round with longer runs
        // (with shorter K, fewer waves per workgroup and as many more workgroups)
        const int mblocks = int((M + 15) / 16);
        int share = 256 * (kNW3Max / NW) / mblocks;
        if (share < 1) share = 1;
        groups = p.tiles < share ? p.tiles : share;
        grid.x = unsigned(groups);
        // K in one pass: the stream form.  Tiles per item as for the 2-bit stream kernel: runs
        // of up to 3 tiles are one item, a run of 4 goes as 2 + 2, longer runs in items of 3.
        const int run = (p.tiles + groups - 1) / groups;
        int T = run <= 3 ? run : (run == 4 ? 2 : 3);
        if (T > NW) T = NW;                                // the epilogue gives every thread at most one output quad
        p.groups = groups;
        Kernel3Fn fn = pick3_stream(T);
        const hipError_t e = raise(fn, 1, T);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(fn, grid, dim3(NW * 64), size_t(NW) * kWave3Lds + kLutBytes, s, p);
        return hipGetLastError();
    }
    int T = (p.tiles + groups - 1) / groups;
    if (T > kT3Max) { T = kT3Max; groups = (p.tiles + T - 1) / T; }
    p.groups = groups;
    grid.x = unsigned(groups);
    Kernel3Fn fn = pick3(T);
    const hipError_t e = raise(fn, 0, T);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(fn, grid, dim3(NW * 64), size_t(NW) * kWave3Lds + kLutBytes, s, p);
    return hipGetLastError();
}

}  // namespace tl
