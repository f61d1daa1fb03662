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
//    c = w + 1 the result is sum_k x_k c_k - sum_k x_k; the second sum comes from one more
//    group of MFMAs per wave whose 16-row operand is a constant, and seeds the accumulator.
//  * Split-K partial tiles of the NW waves are added in a fixed order through LDS, scaled
//    by gamma, rounded to fp16 (RNE) and stored.  No atomics: results are deterministic.
//  * One launch can carry up to 16 independent jobs (a job = one matrix and at most 16
//    activation rows); a workgroup finds its job from its index.  Grouped launches use
//    4-wave groups, two per CU, so that one group's wait for HBM overlaps the other's MFMAs.
#include "tl_internal.hpp"

namespace tl {

namespace {

constexpr int kTMax = 4;          // tiles a workgroup keeps in flight
constexpr int kSliceK = 512;      // K elements a wave owns per pass
constexpr int kWaveLds = 16384;   // bytes of LDS per wave: 16 activation rows x 1 KB
constexpr int kMaxJobs = 16;      // jobs per launch

struct GemvJob {                  // 64 bytes, lives in the kernel argument segment
    const __half* x;              // first activation row of this 16-row block
    const uint32_t* W;
    __half* y;                    // first output row of this block
    float gamma;
    int Mrem;                     // 1..16 activation rows
    int N, K;
    int tiles;                    // ceil(N / 16)
    int groups;                   // workgroups that share this job
    int group0;                   // index of the job's first workgroup in the launch
    int slices;                   // ceil(K / 512)
    int mr;                       // staged rows: power of two >= Mrem (surplus rows repeat)
    int pad;
};

struct GemvBatch {
    int count;
    int pad[3];
    GemvJob job[kMaxJobs];
};

// s_waitcnt immediate for "vmcnt <= n" only (gfx9 layout: vmcnt in bits 3:0 and 15:14,
// expcnt 6:4 and lgkmcnt 11:8 left at their maxima, i.e. not waited for).
constexpr int vmcnt_imm(int n)
{
    return (n & 0xF) | ((n >> 4) << 14) | (0x7 << 4) | (0xF << 8);
}

__device__ __forceinline__ f16x8 as_f16x8(u32x4 v)
{
    return __builtin_bit_cast(f16x8, v);
}

#ifdef TL_GEMV_TRACE
__device__ unsigned long long* g_trace;   // [group][wave][16] time stamps, development builds only
#define TL_STAMP(i) do { tl_stamp[i] = __builtin_amdgcn_s_memtime(); } while (0)
#define TL_STAMP_DECL unsigned long long tl_stamp[16] = {}
#define TL_STAMP_FLUSH do { if (lane == 0) for (int i_ = 0; i_ < 16; ++i_) g_trace[(size_t(blockIdx.x) * 8 + wave) * 16 + i_] = tl_stamp[i_]; } while (0)
#else
#define TL_STAMP(i) do { } while (0)
#define TL_STAMP_DECL do { } while (0)
#define TL_STAMP_FLUSH do { } while (0)
#endif

// T: tiles per workgroup; tile t of group g (within its job) is g + t * groups.
template <int T>
__global__ void __launch_bounds__(512)
gemv_kernel(GemvBatch b)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int NW = blockDim.x >> 6;
    unsigned char* const my_lds = lds_raw + wave * kWaveLds;
    TL_STAMP_DECL;
    TL_STAMP(0);

    int ji = 0;
    while (ji + 1 < b.count && int(blockIdx.x) >= b.job[ji + 1].group0) ++ji;
    const GemvJob& J = b.job[ji];
    const int grp = int(blockIdx.x) - J.group0;
    const int groups = J.groups, tiles = J.tiles, slices = J.slices;
    const int Mrem = J.Mrem, MR = J.mr;
    const int K = J.K, N = J.N;
    const uint32_t row_bytes = uint32_t(K) >> 2;
    const int chunks = K >> 6;                 // 64-weight (16-byte) chunks per row

    // ---- coalesced load mapping: 8 lanes per 128-byte line, 8 rows per instruction ----
    const int lr = lane >> 3;                  // row within the half tile
    const int lc = lane & 7;                   // chunk within the slice
    // ---- MFMA mapping: lane (i, g) = (row / activation column, k group) -----------------
    const int mi = lane & 15;
    const int mg = lane >> 4;
    const int xrow = mi & (MR - 1);            // staged activation row this lane's column reads

    // LDS offsets (bytes, relative to my_lds); immediates add the row / tile / half part
    const uint32_t xr_off = uint32_t(xrow) * 1024u + uint32_t(mg) * 128u;  // + ((c ^ (xrow & 7)) << 4)
    const uint32_t ww_off = uint32_t(lr) * 128u + (uint32_t(lc ^ lr) << 4);
    const uint32_t wr_off0 = uint32_t(mi) * 128u + (uint32_t((mg) ^ (mi & 7)) << 4);
    const uint32_t wr_off1 = uint32_t(mi) * 128u + (uint32_t((4 + mg) ^ (mi & 7)) << 4);

    const unsigned char* const Wb = reinterpret_cast<const unsigned char*>(J.W);
    const unsigned char* const xb = reinterpret_cast<const unsigned char*>(J.x);

    u32x4 wreg[T][2];
    const bool ragged_n = (N & 15) != 0;
    auto issue_w = [&](int t, int slice) {
        int tile = grp + t * groups;
        if (tile >= tiles) tile = tiles - 1;               // loaded again, never used
        int chunk = slice * 8 + lc;
        if (chunk >= chunks) chunk = 0;                    // multiplied by zero activations
        const unsigned char* tb = Wb + size_t(tile) * 16u * row_bytes;
        uint32_t off0 = uint32_t(lr) * row_bytes + uint32_t(chunk) * 16u;
        uint32_t off1 = off0 + 8u * row_bytes;
        if (ragged_n && tile == tiles - 1) {               // scalar branch: rows past N read row N-1
            const int last = N - 1 - tile * 16;
            off0 = uint32_t(lr < last ? lr : last) * row_bytes + uint32_t(chunk) * 16u;
            off1 = uint32_t(lr + 8 < last ? lr + 8 : last) * row_bytes + uint32_t(chunk) * 16u;
        }
        wreg[t][0] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tb + off0));
        wreg[t][1] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tb + off1));
    };

    // Activation rows go straight from global memory into the LDS staging area (LDS-DMA, no
    // registers): one instruction per staged row, lane l fetches the 16-byte piece
    // l ^ (r & 7) of the slice and the hardware drops it at slot l, which is the swizzled
    // layout the operand set-up reads.  Rows past Mrem repeat row Mrem-1; lanes past K
    // store zeros instead (their weights are whatever chunk 0 holds).
    auto issue_x = [&](int slice) {
        for (int r = 0; r < MR; ++r) {
            const int rr = r < Mrem ? r : Mrem - 1;
            const int kx = slice * kSliceK + ((lane ^ (r & 7)) << 3);
            if (kx < K) {
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)(xb + size_t(rr) * K * 2 + uint32_t(kx) * 2u),
                    (__attribute__((address_space(3))) void*)(my_lds + r * 1024),
                    16, 0, 0);
            } else {
                *reinterpret_cast<u32x4*>(my_lds + r * 1024 + (uint32_t(lane) << 4)) = u32x4{0u, 0u, 0u, 0u};
            }
        }
    };

    f32x4 part[T];
#pragma unroll
    for (int t = 0; t < T; ++t) part[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Activations go first: they are short L2 hits, and the loads of one wave return in
    // order, so the weight stream queued behind them overlaps the operand set-up below.
    int slice = wave;
    if (slice < slices) {
        issue_x(slice);
#pragma unroll
        for (int t = 0; t < T; ++t) issue_w(t, slice);
        TL_STAMP(1);
        // The compiler does not track LDS-DMA: wait by hand until only the 2T weight loads
        // issued after the activation rows are outstanding (loads of a wave return in order).
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * T));
        TL_STAMP(2);
    }

    for (; slice < slices; slice += NW) {                  // wave-uniform trip count
        const bool more = (slice + NW) < slices;
        // ---------------- activations of this slice -> MFMA B registers ----------------
        // staging layout: row r, 16-byte piece P at slot P ^ (r & 7)
        // breg[h][wd][e]: (x[k], x[k + 8]) with k = slice0 + 64 (4h + g) + 16 wd + e
        uint32_t breg[2][4][8];
        {
            const uint32_t sw = uint32_t(xrow & 7);
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int wd = 0; wd < 4; ++wd) {
                    const u32x4 lo = *reinterpret_cast<const u32x4*>(
                        my_lds + xr_off + h * 512 + ((uint32_t(2 * wd) ^ sw) << 4));
                    const u32x4 hi = *reinterpret_cast<const u32x4*>(
                        my_lds + xr_off + h * 512 + ((uint32_t(2 * wd + 1) ^ sw) << 4));
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        breg[h][wd][2 * r] = __builtin_amdgcn_perm(hi[r], lo[r], 0x05040100u);
                        breg[h][wd][2 * r + 1] = __builtin_amdgcn_perm(hi[r], lo[r], 0x07060302u);
                    }
                }
        }
        // nsx[r] = -2^-20 sum_k x[m][k] over the slice, in the layout of an accumulator:
        // an MFMA whose 16-row operand is the constant -2^-20 in every position.
        f32x4 nsx = f32x4{0.f, 0.f, 0.f, 0.f};
        {
            const uint32_t c = 0x80108010u;               // fp16 pair of -2^-20 (subnormal 0x0010, sign set)
            const u32x4 a = u32x4{c, c, c, c};
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const u32x4 bb = u32x4{breg[h][0][e], breg[h][1][e], breg[h][2][e], breg[h][3][e]};
                    nsx = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(a), as_f16x8(bb), nsx, 0, 0, 0);
                }
        }
        TL_STAMP(3);
        // ---------------- per tile: turn through LDS, decode, MFMA -----------------------
        // The staging rows are dead once breg is built, so region t (2 KB) reuses them; LDS
        // operations of one wave execute in order.
#pragma unroll
        for (int t = 0; t < T; ++t) {
            unsigned char* const reg_t = my_lds + t * 2048;
            *reinterpret_cast<u32x4*>(reg_t + ww_off) = wreg[t][0];
            *reinterpret_cast<u32x4*>(reg_t + 1024 + ww_off) = wreg[t][1];
            if (more) issue_w(t, slice + NW);              // refill for the next pass
            if (grp + t * groups < tiles) {                // scalar: tiles past the end are skipped
                // acc[0] starts from -2^-20 sum x: with the 2^20 below it carries the "-1" of c = w + 1
                f32x4 acc[3] = {nsx, f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const u32x4 wv = *reinterpret_cast<const u32x4*>(reg_t + (h ? wr_off1 : wr_off0));
                    // element e of each half-word is moved to mantissa bits 4..9 (position
                    // class 2, 3 or 4): e = 0..2 by << 4, e = 3..5 by >> 2, e = 6..7 by >> 8
                    const u32x4 sh[3] = {wv << 4, wv >> 2, wv >> 8};
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int j = e % 3;                        // accumulator: class j + 2
                        const uint32_t mask = 0x00300030u << (2 * j);
                        const u32x4 a = sh[e / 3] & mask;
                        const u32x4 bb = u32x4{breg[h][0][e], breg[h][1][e], breg[h][2][e], breg[h][3][e]};
                        acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(a), as_f16x8(bb), acc[j], 0, 0, 0);
                    }
                }
                // fp16 bits c << (2j + 4) are the subnormal c 4^(j+2) 2^-24: undo with 2^(20 - 2j)
                part[t] += acc[0] * 1048576.f + acc[1] * 262144.f + acc[2] * 65536.f;
            }
            TL_STAMP(4 + t);
        }
        // The staging rows share LDS with the tile regions, so the next slice's activations
        // can only be fetched once the last tile has been read.
        if (more) {
            issue_x(slice + NW);
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));       // behind the prefetched weights
        }
    }

    // ---- split-K reduction across the waves, epilogue -----------------------------------
    // Layout [t][wave][lane] of f32x4 in LDS (reuses the staging space after a barrier).
    TL_STAMP(12);
    __syncthreads();
    TL_STAMP(13);
    f32x4* red = reinterpret_cast<f32x4*>(lds_raw);
#pragma unroll
    for (int t = 0; t < T; ++t) red[(t * NW + wave) * 64 + lane] = part[t];
    __syncthreads();
    const float gamma = J.gamma;
    for (int item = threadIdx.x; item < T * 64; item += blockDim.x) {
        const int t = item >> 6;
        const int l = item & 63;
        const int tile = grp + t * groups;
        if (tile >= tiles) continue;
        f32x4 v[8];
#pragma unroll
        for (int w = 0; w < 8; ++w)                         // all reads in flight, then a fixed-order sum
            v[w] = (w < NW) ? red[(t * NW + w) * 64 + l] : f32x4{0.f, 0.f, 0.f, 0.f};
        const f32x4 s = ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
        const int n = tile * 16 + 4 * (l >> 4);
        if ((l & 15) < Mrem) {
            __half* dst = J.y + size_t(l & 15) * N + n;
            if (n + 3 < N && (N & 3) == 0) {                // four consecutive n: one 8-byte store
                const f16x2 lo = {(_Float16)(gamma * s[0]), (_Float16)(gamma * s[1])};
                const f16x2 hi = {(_Float16)(gamma * s[2]), (_Float16)(gamma * s[3])};
                *reinterpret_cast<u32x2*>(dst) = u32x2{__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (n + r < N) dst[r] = __float2half_rn(gamma * s[r]);
            }
        }
    }
    TL_STAMP(14);
    TL_STAMP_FLUSH;
}

using KernelFn = void (*)(GemvBatch);

KernelFn pick_kernel(int T)
{
    switch (T) {
        case 1: return gemv_kernel<1>;
        case 2: return gemv_kernel<2>;
        case 3: return gemv_kernel<3>;
        default: return gemv_kernel<4>;
    }
}

int pow2_at_least(int v)
{
    int r = 1;
    while (r < v) r *= 2;
    return r;
}

// Launch one batch (<= kMaxJobs jobs with group0 / groups filled in).
hipError_t launch_batch(GemvBatch& b, int T, int NW, int total_groups, hipStream_t s)
{
    KernelFn fn = pick_kernel(T);
    // Groups of 5 or more waves need more than the default 64 KB of dynamic LDS; the
    // attribute is set once per kernel instance (idempotent, so a race only repeats it).
    static bool lds_raised[kTMax + 1];
    if (!lds_raised[T]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 8 * kWaveLds);
        if (e != hipSuccess) return e;
        lds_raised[T] = true;
    }
    hipLaunchKernelGGL(fn, dim3(total_groups), dim3(NW * 64), size_t(NW) * kWaveLds, s, b);
    return hipGetLastError();
}

}  // namespace

bool gemv_supports(int64_t M, int64_t N, int64_t K)
{
    return M >= 1 && N >= 1 && K >= 64 && (K % 64) == 0 && K <= (int64_t(1) << 24) &&
           N <= (int64_t(1) << 24) && M <= (int64_t(1) << 20);
}

hipError_t launch_gemv_jobs(const GemmDesc* jobs, int count, hipStream_t s)
{
    // A user job with M > 16 becomes ceil(M / 16) kernel jobs (blocks of 16 activation rows).
    // One job alone gets 8-wave groups, one per CU, each holding up to 4 tiles; several jobs
    // in one launch get 4-wave groups (two passes over K = 4096), two groups per CU, so that
    // one group's wait for HBM overlaps the other's arithmetic (measured best of the
    // (waves, tiles, groups) settings tried on the decode sweep).
    int64_t blocks_total = 0;
    for (int i = 0; i < count; ++i) blocks_total += (jobs[i].M + 15) / 16;
    const bool grouped = blocks_total > 1;
    const int nw_cap = grouped ? 4 : 8;
    const int t_cap = kTMax;
    const int group_cap = 256;

    GemvBatch b;
    b.count = 0;
    int total_groups = 0, Tmax = 1, NW = 1;
    auto flush = [&]() -> hipError_t {
        if (b.count == 0) return hipSuccess;
        hipError_t e = launch_batch(b, Tmax, NW, total_groups, s);
        b.count = 0; total_groups = 0; Tmax = 1; NW = 1;
        return e;
    };
    for (int i = 0; i < count; ++i) {
        const GemmDesc& d = jobs[i];
        for (int64_t m0 = 0; m0 < d.M; m0 += 16) {
            GemvJob j;
            j.x = d.x + m0 * d.K;
            j.W = d.W;
            j.y = d.y + m0 * d.N;
            j.gamma = d.gamma;
            j.Mrem = int(d.M - m0 < 16 ? d.M - m0 : 16);
            j.N = int(d.N); j.K = int(d.K);
            j.tiles = int((d.N + 15) / 16);
            j.slices = int((d.K + kSliceK - 1) / kSliceK);
            j.mr = pow2_at_least(j.Mrem);
            j.pad = 0;
            int groups = j.tiles < group_cap ? j.tiles : group_cap;
            int T = (j.tiles + groups - 1) / groups;
            if (T > t_cap) { T = t_cap; groups = (j.tiles + T - 1) / T; }
            j.groups = groups;
            j.group0 = total_groups;
            total_groups += groups;
            if (T > Tmax) Tmax = T;
            const int nw = j.slices < nw_cap ? j.slices : nw_cap;
            if (nw > NW) NW = nw;
            b.job[b.count++] = j;
            if (b.count == kMaxJobs) {
                hipError_t e = flush();
                if (e != hipSuccess) return e;
            }
        }
    }
    return flush();
}

hipError_t launch_gemv(const __half* x, const uint32_t* Wp, float gamma, __half* y,
                       int64_t M, int64_t N, int64_t K, hipStream_t s)
{
    GemmDesc d{x, Wp, y, gamma, M, N, K};
    return launch_gemv_jobs(&d, 1, s);
}

}  // namespace tl
