// LDS-tiled fp16 MFMA kernel for large M (prefill): Y = X (gamma What)^T of App. B, where the
// 2-bit codes of Sec. 3.1 are decoded to fp16 -1/0/+1 on their way into LDS.
//
// A workgroup of 4 waves (2 x 2) owns a BM x BN tile of Y (128 x 256 or 128 x 128; at least two
// groups are resident per CU) and walks K in steps of 64.
// Per step: the X tile [BM][64] is copied into LDS as it is; each packed row slice (one
// dwordx4 = 64 codes) is decoded in registers and written as 64 fp16 values; then every
// wave runs v_mfma_f32_32x32x16_f16 over its (BM/2) x (BN/2) sub-tile, X as the 32-row
// operand and W as the 32-column operand, so that a lane's accumulator registers hold
// consecutive n of one output row.  The loads of step s+1 are issued before the MFMAs of
// step s (register prefetch, one LDS buffer, two barriers per step).
//
// Decode (per 32-bit word, 16 codes): `(w & (3 << 2j | 3 << (2j+16))) | 0x64006400` is the
// fp16 pair (1024 + 4^j c_j, 1024 + 4^j c_{j+8}); one packed fma with 4^-j and
// -(1024 4^-j + 1) turns it into (c_j - 1, c_{j+8} - 1) exactly.  Codes 5..7 come from the
// word shifted right by 10.  v_perm_b32 then pairs neighbours so that LDS holds k in order.
#include "tl_internal.hpp"

namespace tl {

namespace {

constexpr int BK = 64;                 // K elements per step
constexpr int LDS_ROW = BK + 8;        // halves per LDS row: 144 bytes, keeps b128 reads conflict-free

struct MfmaParams {
    const __half* x;
    const uint32_t* W;
    __half* y;
    float gamma;
    int M, N, K;
    int tiles_m, tiles_n;
};

__device__ __forceinline__ uint32_t pk_fma(uint32_t a, uint32_t b, uint32_t c)
{
    const f16x2 r = __builtin_elementwise_fma(__builtin_bit_cast(f16x2, a), __builtin_bit_cast(f16x2, b),
                                              __builtin_bit_cast(f16x2, c));
    return __builtin_bit_cast(uint32_t, r);
}

// 16 codes of one word -> 16 fp16 weights in k order, as 8 packed pairs (k, k+1).
__device__ __forceinline__ void decode_word(uint32_t w, uint32_t (&out)[8])
{
    // scale 4^-j and offset -(1024 4^-j + 1) as fp16 pairs, j = 0..4
    constexpr uint32_t kScale[5] = {0x3C003C00u, 0x34003400u, 0x2C002C00u, 0x24002400u, 0x1C001C00u};
    constexpr uint32_t kOff[5] = {0xE401E401u, 0xDC04DC04u, 0xD410D410u, 0xCC40CC40u, 0xC500C500u};
    uint32_t p[8];                                     // p[j] = (w_j, w_{j+8})
    const uint32_t ws = w >> 10;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int jj = (j < 5) ? j : j - 5;
        const uint32_t src = (j < 5) ? w : ws;
        const uint32_t t = (src & (0x00030003u << (2 * jj))) | 0x64006400u;
        p[j] = pk_fma(t, kScale[jj], kOff[jj]);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        out[r] = __builtin_amdgcn_perm(p[2 * r + 1], p[2 * r], 0x05040100u);       // (w_2r, w_2r+1)
        out[4 + r] = __builtin_amdgcn_perm(p[2 * r + 1], p[2 * r], 0x07060302u);   // (w_2r+8, w_2r+9)
    }
}

template <int BM, int BN>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 8)))
mfma_kernel(MfmaParams p)
{
    constexpr int PD = 1;                              // steps of global loads in flight
    constexpr int WM = BM / 2, WN = BN / 2;            // per-wave sub-tile
    constexpr int FM = WM / 32, FN = WN / 32;          // 32x32 fragments per wave
    constexpr int XL = BM * 8 / 256;                   // dwordx4 loads of X per thread and step
    constexpr int WL = (BN + 255) / 256;               // packed rows per thread and step
    __shared__ __attribute__((aligned(16))) _Float16 As[BM * LDS_ROW];
    __shared__ __attribute__((aligned(16))) _Float16 Bs[BN * LDS_ROW];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // XCD-aware tile order: consecutive workgroup ids go to different XCDs (8 of them), so a
    // group's position inside its XCD picks neighbouring tiles that share a W column block.
    const int total = p.tiles_m * p.tiles_n;
    int id = blockIdx.x;
    {
        const int per_xcd = (total + 7) / 8;
        const int remapped = (id & 7) * per_xcd + (id >> 3);
        id = (remapped < total && (total & 7) == 0) ? remapped : id;
    }
    const int tn = id / p.tiles_m;
    const int tm = id - tn * p.tiles_m;
    const int m_base = tm * BM;
    const int n_base = tn * BN;
    const int K = p.K;
    const int row_words = K >> 4;

    // ---- global load plan ---------------------------------------------------------------
    // X: thread t copies, for i < XL, the 16 bytes at row (t/8 + 32 i), halves 8 (t%8) .. +7
    const int xr = tid >> 3, xc = tid & 7;
    const __half* xsrc[XL];
#pragma unroll
    for (int i = 0; i < XL; ++i) {
        int m = m_base + xr + 32 * i;
        if (m >= p.M) m = p.M - 1;                        // rows past M are computed, not stored
        xsrc[i] = p.x + size_t(m) * K + xc * 8;
    }
    // W: thread t owns packed row t (+256 i) of the tile
    const uint32_t* wsrc[WL];
#pragma unroll
    for (int i = 0; i < WL; ++i) {
        int n = n_base + tid + 256 * i;
        if (n >= p.N) n = p.N - 1;
        wsrc[i] = p.W + size_t(n) * row_words;
    }
    const bool w_active = (WL > 1) || (tid < BN);

    // Register ring of PD steps: the loads of step s + PD are issued while step s is computed,
    // because one step of MFMAs (about 0.9 us) is shorter than a trip to L2 / Infinity Cache.
    u32x4 xreg[PD][XL];
    u32x4 wreg[PD][WL];
    auto load_step = [&](int slot, int k0) {
#pragma unroll
        for (int i = 0; i < XL; ++i) xreg[slot][i] = *reinterpret_cast<const u32x4*>(xsrc[i] + k0);
        if (w_active) {
#pragma unroll
            for (int i = 0; i < WL; ++i) wreg[slot][i] = *reinterpret_cast<const u32x4*>(wsrc[i] + (k0 >> 4));
        }
    };
    auto store_step = [&](int slot) {
#pragma unroll
        for (int i = 0; i < XL; ++i)
            *reinterpret_cast<u32x4*>(&As[(xr + 32 * i) * LDS_ROW + xc * 8]) = xreg[slot][i];
        if (w_active) {
#pragma unroll
            for (int i = 0; i < WL; ++i) {
                _Float16* dst = &Bs[(tid + 256 * i) * LDS_ROW];
#pragma unroll
                for (int wd = 0; wd < 4; ++wd) {
                    uint32_t o[8];
                    decode_word(wreg[slot][i][wd], o);
                    *reinterpret_cast<u32x4*>(dst + wd * 16) = u32x4{o[0], o[1], o[2], o[3]};
                    *reinterpret_cast<u32x4*>(dst + wd * 16 + 8) = u32x4{o[4], o[5], o[6], o[7]};
                }
            }
        }
    };

    f32x16 acc[FM][FN];
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    // fragment addresses: lane (i = lane % 32, kg = lane / 32) reads 8 halves of row i
    const int fi = lane & 31, fk = (lane >> 5) * 8;
    const _Float16* a_frag = &As[(wm * WM + fi) * LDS_ROW + fk];
    const _Float16* b_frag = &Bs[(wn * WN + fi) * LDS_ROW + fk];

#pragma unroll
    for (int d = 0; d < PD; ++d)
        if (d * BK < K) load_step(d, d * BK);
    for (int kb = 0; kb < K; kb += PD * BK) {
#pragma unroll
      for (int d = 0; d < PD; ++d) {
        const int k0 = kb + d * BK;
        if (k0 >= K) break;
        store_step(d);
        __syncthreads();
        if (k0 + PD * BK < K) load_step(d, k0 + PD * BK);
#pragma unroll
        for (int ks = 0; ks < BK; ks += 16) {
            f16x8 af[FM], bf[FN];
#pragma unroll
            for (int a = 0; a < FM; ++a)
                af[a] = *reinterpret_cast<const f16x8*>(a_frag + a * 32 * LDS_ROW + ks);
#pragma unroll
            for (int b = 0; b < FN; ++b)
                bf[b] = *reinterpret_cast<const f16x8*>(b_frag + b * 32 * LDS_ROW + ks);
#pragma unroll
            for (int a = 0; a < FM; ++a)
#pragma unroll
                for (int b = 0; b < FN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[a], bf[b], acc[a][b], 0, 0, 0);
        }
        __syncthreads();
      }
    }

    // ---- epilogue: y[m][n] = fp16(gamma * acc) ---------------------------------------------
    // D[i][j] of a 32x32 fragment: j = lane % 32, i = 8 (r / 4) + 4 (lane / 32) + r % 4.
    const int col = lane & 31;
    const int rsub = (lane >> 5) * 4;
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b) {
            const int n = n_base + wn * WN + b * 32 + col;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m_base + wm * WM + a * 32 + 8 * (r >> 2) + rsub + (r & 3);
                if (m < p.M && n < p.N) p.y[size_t(m) * p.N + n] = __float2half_rn(p.gamma * acc[a][b][r]);
            }
        }
}

}  // namespace

bool mfma_supports(int64_t M, int64_t N, int64_t K)
{
    return M >= 1 && N >= 1 && K >= 64 && (K % 64) == 0 && K <= (int64_t(1) << 24) &&
           M <= (int64_t(1) << 24) && N <= (int64_t(1) << 24);
}

hipError_t launch_mfma(const __half* x, const uint32_t* Wp, float gamma, __half* y,
                       int64_t M, int64_t N, int64_t K, hipStream_t s)
{
    MfmaParams p;
    p.x = x; p.W = Wp; p.y = y; p.gamma = gamma;
    p.M = int(M); p.N = int(N); p.K = int(K);
    // 128 x 256 tiles keep two workgroups resident per CU (128 accumulator registers per
    // wave), so one group's decode / barrier phase hides behind the other's MFMAs: measured
    // 1.0 PFLOP/s at M = 2048 against 0.87 for one resident 256 x 256 group.  Small M takes
    // 128 x 128 tiles to give every CU work.
    if (M > 256) {
        p.tiles_m = int((M + 127) / 128); p.tiles_n = int((N + 255) / 256);
        hipLaunchKernelGGL((mfma_kernel<128, 256>), dim3(p.tiles_m * p.tiles_n), dim3(256), 0, s, p);
    } else {
        p.tiles_m = int((M + 127) / 128); p.tiles_n = int((N + 127) / 128);
        hipLaunchKernelGGL((mfma_kernel<128, 128>), dim3(p.tiles_m * p.tiles_n), dim3(256), 0, s, p);
    }
    return hipGetLastError();
}

}  // namespace tl
