// LDS-tiled fp16 MFMA kernel for large M (prefill): Y = X (gamma What)^T of App. B, where the
// 2-bit codes of Sec. 3.1 are decoded to fp16 -1/0/+1 in registers, right before the matrix
// instruction that consumes them.
//
// A workgroup of 4 waves owns a 128 x (4 NW) tile of Y: the waves sit side by side along N,
// NW = 64 or 32 columns each, and all four use the same 128 rows of X.  K is walked in steps
// of 64.
//
//  * W stays packed all the way into LDS.  Per step a wave needs 16 bytes (64 codes) of each
//    of its NW rows: one `global_load_lds_dwordx4` drops them into a wave-private ring of
//    WSTAGES = 4 stages, three steps ahead, with no registers and no barrier involved.  A lane
//    (column i, k half g) reads its row's 16 bytes back (one ds_read_b128 per 32 columns and
//    step, issued one step early) and decodes, per 16-k block, the half-word it needs:
//    `(w >> 8g) & (3 << 2j | 3 << (2j+16)) | 0x64006400` is the fp16 pair (1024 + 4^j c_j', 1024 + 4^j c_j'+8), j' = 4g + j,
//    and one packed fma with 4^-j and -(1024 4^-j + 1) turns it into (c - 1, c - 1) exactly:
//    2 VALU operations per operand register, and an operand register set feeds 4 MFMAs.
//  * That pairs k with k + 8 inside every 16-k block.  The matrix instruction does not care
//    in which order k runs as long as both operands agree, so X is stored to LDS in the same
//    order: on its way from global memory through registers (prefetched XS = 4 steps ahead) each
//    thread interleaves the two 8-k pieces of a block with v_perm_b32.  X is double-buffered
//    in LDS (padded rows, conflict-free b128 reads), so a step costs one barrier.
//  * Every wave runs v_mfma_f32_32x32x16_f16 over a 128 x NW sub-tile (4 x NW/32 fragments),
//    X as the 32-row operand and W as the 32-column operand.
//  * Launches of at most one 128 x 128 tile per CU use two such sets of 4 waves per workgroup,
//    each with half of the K steps (SPLIT below).
#include "tl_internal.hpp"

namespace tl {

namespace {

constexpr int BK = 64;                 // K elements per step
constexpr int BM = 128;                // rows of X per workgroup
constexpr int XROW = 144;              // bytes per X row in LDS: 128 + 16, keeps b128 reads conflict-free
constexpr int XBUF = BM * XROW;        // one X buffer
constexpr int WSTAGES = 4;             // steps of packed W in flight per wave
constexpr int WSTAGE = 1024;           // bytes per stage: 64 rows x 16 bytes

constexpr int kWideMin = 129;          // 128 x 256 tiles from this many of them on (measured crossover)
constexpr bool kSplit = true;          // 128 x 128 tiles: two sets of waves per tile when K allows

struct MfmaParams {
    const __half* x;
    const uint32_t* W;
    __half* y;
    float gamma;
    int M, N, K;
    int tiles_m, tiles_n;
};

// s_waitcnt immediate for "vmcnt <= n" only (gfx9 layout)
constexpr int vm_imm(int n)
{
    return (n & 0xF) | ((n >> 4) << 14) | (0x7 << 4) | (0xF << 8);
}

__device__ __forceinline__ uint32_t pk_fma(uint32_t a, uint32_t b, uint32_t c)
{
    const f16x2 r = __builtin_elementwise_fma(__builtin_bit_cast(f16x2, a), __builtin_bit_cast(f16x2, b),
                                              __builtin_bit_cast(f16x2, c));
    return __builtin_bit_cast(uint32_t, r);
}

// The 8 codes (j, j + 8), j = 0..3, of a half-word-shifted packed word -> 4 fp16 pairs (w_j, w_j+8).
__device__ __forceinline__ f16x8 decode_half(uint32_t hw, uint32_t k1024)
{
    constexpr uint32_t kScale[4] = {0x3C003C00u, 0x34003400u, 0x2C002C00u, 0x24002400u};   // 4^-j
    constexpr uint32_t kOff[4] = {0xE401E401u, 0xDC04DC04u, 0xD410D410u, 0xCC40CC40u};     // -(1024 4^-j + 1)
    u32x4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t t = (hw & (0x00030003u << (2 * j))) | k1024;
        o[j] = pk_fma(t, kScale[j], kOff[j]);
    }
    return __builtin_bit_cast(f16x8, o);
}

// NW: columns of Y per wave (64 or 32); XS: steps of X in flight in registers (even).
// SPLIT = 2: the workgroup has two such sets of 4 waves; set h takes the K steps 2 t + h (K a
// multiple of 128), with X buffers and W rings of its own, and the sets' sums are added through
// LDS at the end.  For launches of at most one tile per CU, where a lone set leaves each SIMD
// with one wave that waits out every load, LDS round trip and barrier of a step.
template <int SPLIT>
constexpr int mfma_lds_bytes() { return SPLIT * (2 * XBUF + 4 * WSTAGES * WSTAGE); }

template <int NW, int XS, int SPLIT>
__global__ void __launch_bounds__(256 * SPLIT) __attribute__((amdgpu_waves_per_eu(2, 2)))
mfma_kernel(MfmaParams p)
{
    constexpr int FM = BM / 32;                        // 4 fragments down
    constexpr int FN = NW / 32;                        // 2 or 1 fragments across
    constexpr int BN = 4 * NW;
    static_assert(SPLIT == 1 || (SPLIT == 2 && FN == 1), "the sums of the second set go through the X buffers");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_all[];

    const int set = SPLIT == 2 ? __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 8) : 0;
    const int tid = threadIdx.x & 255;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);        // within the set
    unsigned char* const Xs = lds_all + set * (2 * XBUF);
    unsigned char* const Ws = lds_all + SPLIT * (2 * XBUF) + set * (4 * WSTAGES * WSTAGE);

    // XCD-aware tile order.  Consecutive workgroup ids go to different XCDs (8 of them, each with an
    // L2 of its own), so workgroup id is the (id / 8)-th of XCD id % 8.  Each XCD owns a region of
    // the tile grid and walks it in bands of 4 row blocks, column block by column block: the 64
    // workgroups that are resident on an XCD at a time then form 4 row blocks x 16 column blocks, so
    // that a block of X is fetched into that L2 once for 16 tiles and a block of W once for 4
    // (measured against XCD = column bands over all rows: +1 % at 2048 x 14336, +5 to 6 % at
    // 4096 x 12288 and 4096 x 14336, +4 % at 2048 x 4096 x 11008; the chip is power-limited here,
    // and bytes that do not cross the fabric are power for the matrix pipes).
    const int total = p.tiles_m * p.tiles_n;
    int tn, tm;
    {
        const int x = int(blockIdx.x) & 7, q = int(blockIdx.x) >> 3;
        int rx = 0, xpb = 1;                            // row blocks per XCD region, XCDs side by side per band of rows
        if ((p.tiles_m & 31) == 0) {
            rx = p.tiles_m >> 3;
        } else if (p.tiles_m == 4 || p.tiles_m == 8 || p.tiles_m == 16) {
            rx = 4;
            xpb = 8 / (p.tiles_m >> 2);
        }
        if (rx != 0 && p.tiles_n % xpb == 0) {
            const int cx = p.tiles_n / xpb;             // column blocks per region
            const int band = x / xpb, part = x - band * xpb;
            const int s4 = q / (4 * cx), r = q - s4 * (4 * cx);
            tn = part * cx + (r >> 2);
            tm = band * rx + 4 * s4 + (r & 3);
        } else {
            // any other grid: XCD x takes the x-th eighth of the tiles in column-major order
            int id = blockIdx.x;
            const int per_xcd = (total + 7) / 8;
            const int remapped = x * per_xcd + q;
            id = (remapped < total && (total & 7) == 0) ? remapped : id;
            tn = id / p.tiles_m;
            tm = id - tn * p.tiles_m;
        }
    }
    const int m_base = tm * BM;
    const int n_base = tn * BN + wave * NW;            // this wave's first column
    const int K = p.K;
    const int steps = K / BK / SPLIT;                  // steps of this set
    // step t of this set as a step of K; past the end: a valid one, loaded and never used
    auto kstep = [&](int t) {
        if (t >= steps) t = steps - 1;
        return t * SPLIT + set;
    };

    // ---- X: thread t copies the 64 bytes (32 k) at row t / 2, half t % 2 of every step --------
    const int xr = tid >> 1, xh = tid & 1;
    const unsigned char* xsrc;
    {
        int m = m_base + xr;
        if (m >= p.M) m = p.M - 1;                     // rows past M are computed, not stored
        xsrc = reinterpret_cast<const unsigned char*>(p.x + size_t(m) * K) + xh * 64;
    }
    unsigned char* const xdst = Xs + xr * XROW + xh * 64;
    typedef const __attribute__((address_space(1))) u32x4* gptr;
    u32x4 xreg[XS][4];                                  // XS steps in flight
    auto load_x = [&](int slot, int step) {
        const unsigned char* src = xsrc + size_t(kstep(step)) * (BK * 2);
#pragma unroll
        for (int i = 0; i < 4; ++i) xreg[slot][i] = *(gptr)(src + 16 * i);
    };
    // pieces (k 0..7 | k 8..15) of a 16-k block -> (k0 k8 k1 k9 k2 k10 k3 k11 | k4 k12 .. k7 k15)
    auto store_x = [&](int slot, int buf) {
        unsigned char* dst = xdst + buf * XBUF;
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
            const u32x4 d = xreg[slot][2 * blk], e = xreg[slot][2 * blk + 1];
            u32x4 g0, g1;
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                g0[2 * r] = __builtin_amdgcn_perm(e[r], d[r], 0x05040100u);
                g0[2 * r + 1] = __builtin_amdgcn_perm(e[r], d[r], 0x07060302u);
                g1[2 * r] = __builtin_amdgcn_perm(e[2 + r], d[2 + r], 0x05040100u);
                g1[2 * r + 1] = __builtin_amdgcn_perm(e[2 + r], d[2 + r], 0x07060302u);
            }
            *reinterpret_cast<u32x4*>(dst + blk * 32) = g0;
            *reinterpret_cast<u32x4*>(dst + blk * 32 + 16) = g1;
        }
    };

    // ---- W: lane l fetches the 16 bytes of row n_base + l (NW = 32: lanes 32.. repeat) --------
    unsigned char* const wring = Ws + wave * (WSTAGES * WSTAGE);
    const unsigned char* wsrc;
    {
        int n = n_base + (lane & (NW - 1));
        if (n >= p.N) n = p.N - 1;
        wsrc = reinterpret_cast<const unsigned char*>(p.W) + size_t(n) * (size_t(K) >> 2);
    }
    // The transfer is written out by hand (LDS base in M0, lane l lands at base + 16 l): a
    // transfer the compiler knows of makes it drain the whole memory pipeline before every
    // later LDS access, because it cannot tell that those touch other addresses.  Unknown to
    // it, the transfers only make its own wait counts for the X loads a little stricter.
    const uint32_t wring_addr = uint32_t(uintptr_t((const __attribute__((address_space(3))) unsigned char*)wring));
    auto issue_w = [&](int step) {
        const uint32_t stage = uint32_t(step & (WSTAGES - 1));
        const unsigned char* src = wsrc + size_t(kstep(step)) * 16;
        const uint32_t base = __builtin_amdgcn_readfirstlane(wring_addr + stage * WSTAGE);
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(base) : "memory");   // (m0 is never allocated by the compiler: it sets it right before each of its own uses)
    };

    // Barrier that waits for this wave's LDS traffic only: global loads and W transfers stay in
    // flight across it (__syncthreads would drain them).
    auto lds_barrier = [&]() {
        __builtin_amdgcn_s_waitcnt(0xF | (0x3 << 14) | (0x7 << 4));      // lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
    };

    f32x16 acc[FM][FN];
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    // fragment addresses: lane (i = lane % 32, g = lane / 32)
    const int fi = lane & 31, fg = lane >> 5;
    const unsigned char* const a_frag = Xs + fi * XROW + fg * 16;
    const uint32_t b_addr =                                 // LDS byte address of this lane's row in stage 0
        uint32_t(uintptr_t((const __attribute__((address_space(3))) unsigned char*)(wring + fi * 16)));
    const uint32_t hshift = 8u * uint32_t(fg);
    // The exponent pattern lives in a vector register the compiler cannot see through: with the
    // mask in a scalar register, mask and merge are then one v_and_or_b32 (as two literals they
    // are two instructions, since that encoding takes no literal).
    uint32_t k1024;
    asm volatile("v_mov_b32 %0, 0x64006400" : "=v"(k1024));

    // The packed words of the next step are read from the ring right before the barrier that ends
    // a step.  W of step t: (WSTAGES - 2) steps of 4 X loads and 1 transfer each were issued after
    // it by then.  Hand-written ds_read: for an LDS read it can see, the compiler waits until every
    // LDS-DMA transfer in flight has landed.  Read, wait and barrier are one statement, so that the
    // registers count as written only once the wait is behind them; the wait is for LDS traffic
    // only: global loads and W transfers stay in flight across it (__syncthreads would drain them).
    u32x4 wnext[FN];
    auto read_w_and_barrier = [&](int t) {
        __builtin_amdgcn_s_waitcnt(vm_imm(5 * (WSTAGES - 2)));
        const uint32_t waddr = b_addr + uint32_t(t & (WSTAGES - 1)) * WSTAGE;
        if constexpr (FN == 2) {
            asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:512\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier"
                         : "=&v"(wnext[0]), "=&v"(wnext[1]) : "v"(waddr) : "memory");
        } else {
            asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" : "=&v"(wnext[0]) : "v"(waddr) : "memory");
        }
    };
    // ---- prologue ---------------------------------------------------------------------------
    // Order of the memory operations of a wave, per step: 4 X loads, then 1 W transfer.  The
    // compiler counts the X loads itself; the W transfers (LDS-DMA) are waited for by hand.
    load_x(0, 0);
#pragma unroll
    for (int d = 0; d < WSTAGES - 1; ++d) issue_w(d);
    store_x(0, 0);
#pragma unroll
    for (int d = 1; d <= XS; ++d) load_x(d % XS, d);   // slot j % XS holds X of step j
    read_w_and_barrier(0);

    auto step_body = [&](auto slot_tag, int s) {
        constexpr int SLOT = decltype(slot_tag)::value;        // (s + 1) % XS
        constexpr int PAR = (SLOT + 1) & 1;                    // s & 1 (XS is even)
        // X of step s + 1 (loaded XS steps ago) -> the other buffer; then fetch step s + 1 + XS
        store_x(SLOT, PAR ^ 1);
        load_x(SLOT, s + 1 + XS);
        issue_w(s + WSTAGES - 1);
        const unsigned char* const xb = a_frag + PAR * XBUF;
        u32x4 wq[FN];
#pragma unroll
        for (int b = 0; b < FN; ++b) wq[b] = wnext[b];
        if constexpr (SPLIT == 2) {
            // The two waves of a SIMD belong to the two sets and run in step (same barriers), so
            // neither hides the other's waits: all X fragments of the step are requested up front.
            f16x8 af[4][FM];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int a = 0; a < FM; ++a)
                    af[ks][a] = *reinterpret_cast<const f16x8*>(xb + a * 32 * XROW + ks * 32);
            __builtin_amdgcn_sched_barrier(0);         // or the scheduler moves each read down to its use
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                f16x8 bf[FN];
#pragma unroll
                for (int b = 0; b < FN; ++b) bf[b] = decode_half(wq[b][ks] >> hshift, k1024);
#pragma unroll
                for (int a = 0; a < FM; ++a)
#pragma unroll
                    for (int b = 0; b < FN; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[ks][a], bf[b], acc[a][b], 0, 0, 0);
            }
        } else {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            f16x8 af[FM], bf[FN];
#pragma unroll
            for (int a = 0; a < FM; ++a)
                af[a] = *reinterpret_cast<const f16x8*>(xb + a * 32 * XROW + ks * 32);
#pragma unroll
            for (int b = 0; b < FN; ++b) bf[b] = decode_half(wq[b][ks] >> hshift, k1024);
#pragma unroll
            for (int a = 0; a < FM; ++a)
#pragma unroll
                for (int b = 0; b < FN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[a], bf[b], acc[a][b], 0, 0, 0);
        }
        }
        read_w_and_barrier(s + 1);
    };

    // steps in groups of XS, so that register slots and buffer parity are compile-time
    int s = 0;
    for (; s + XS <= steps; s += XS) {
        step_body(std::integral_constant<int, 1 % XS>{}, s);
        step_body(std::integral_constant<int, 2 % XS>{}, s + 1);
        if constexpr (XS == 4) {
            step_body(std::integral_constant<int, 3>{}, s + 2);
            step_body(std::integral_constant<int, 0>{}, s + 3);
        }
    }
    if (s < steps) { step_body(std::integral_constant<int, 1 % XS>{}, s); ++s; }
    if (s < steps) { step_body(std::integral_constant<int, 2 % XS>{}, s); ++s; }
    if constexpr (XS == 4)
        if (s < steps) { step_body(std::integral_constant<int, 3>{}, s); ++s; }
    __builtin_amdgcn_s_waitcnt(vm_imm(0));             // nothing of this wave's ring is left in flight

    if constexpr (SPLIT == 2) {
        // Every wave is past the barrier of its last step: the X buffers are free.  16 KB per wave.
        float* const red = reinterpret_cast<float*>(lds_all) + wave * (FM * FN * 16 * 64) + lane;
        if (set == 1) {
#pragma unroll
            for (int a = 0; a < FM; ++a)
#pragma unroll
                for (int b = 0; b < FN; ++b)
#pragma unroll
                    for (int r = 0; r < 16; ++r) red[((a * FN + b) * 16 + r) * 64] = acc[a][b][r];
        }
        lds_barrier();
        if (set == 1) return;
#pragma unroll
        for (int a = 0; a < FM; ++a)
#pragma unroll
            for (int b = 0; b < FN; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[a][b][r] += red[((a * FN + b) * 16 + r) * 64];
    }

    // ---- epilogue: y[m][n] = fp16(gamma * acc) ---------------------------------------------
    // D[i][j] of a 32x32 fragment: j = lane % 32, i = 8 (r / 4) + 4 (lane / 32) + r % 4.
    const int col = lane & 31;
    const int rsub = (lane >> 5) * 4;
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b) {
            const int n = n_base + b * 32 + col;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m_base + a * 32 + 8 * (r >> 2) + rsub + (r & 3);
                if (m < p.M && n < p.N) p.y[size_t(m) * p.N + n] = __float2half_rn(p.gamma * acc[a][b][r]);
            }
        }
}

}  // namespace

// Raises the dynamic-LDS limit of the two-set instance on the current device (104 KB).
hipError_t mfma_init()
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&mfma_kernel<32, 4, 2>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, mfma_lds_bytes<2>());
}

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
    p.tiles_m = int((M + BM - 1) / BM);
    // 128 x 256 tiles, two workgroups resident per CU; 128 x 128 tiles while those would leave
    // half of the CUs without work
    const int64_t wide = int64_t(p.tiles_m) * ((N + 255) / 256);
    if (wide >= kWideMin) {
        p.tiles_n = int((N + 255) / 256);
        hipLaunchKernelGGL((mfma_kernel<64, 4, 1>), dim3(p.tiles_m * p.tiles_n), dim3(256), mfma_lds_bytes<1>(), s, p);
    } else if (kSplit && K % (2 * BK) == 0) {
        // at most one tile per CU: two sets of waves per tile, each with half of the K steps
        static bool raised[kMaxDevices];
        const int dev = device_slot();
        if (dev < 0 || !raised[dev]) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&mfma_kernel<32, 4, 2>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, mfma_lds_bytes<2>());
            if (e != hipSuccess) return e;
            if (dev >= 0) raised[dev] = true;
        }
        p.tiles_n = int((N + 127) / 128);
        hipLaunchKernelGGL((mfma_kernel<32, 4, 2>), dim3(p.tiles_m * p.tiles_n), dim3(512), mfma_lds_bytes<2>(), s, p);
    } else {
        p.tiles_n = int((N + 127) / 128);
        hipLaunchKernelGGL((mfma_kernel<32, 4, 1>), dim3(p.tiles_m * p.tiles_n), dim3(256), mfma_lds_bytes<1>(), s, p);
    }
    return hipGetLastError();
}

}  // namespace tl
