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
//  * Decode costs 10 to 11 VALU operations per 16 weights.  `word & (3 << 2j | 3 << (2j+16))`
//    leaves two codes in the mantissa fields of an fp16 pair, i.e. the subnormal numbers
//    c * 4^j * 2^-24 (gfx950 MFMA does not flush fp16 subnormals).  The matrix core aligns
//    products by their exponent FIELDS, so a code low in the mantissa loses accuracy
//    (measured: ~2^-17 relative at j = 0, none at j >= 3).  Shifted copies of the word therefore
//    bring every code to j in {2, 3, 4}: the stream and lean kernels use the word as loaded and
//    two copies (<< 4, >> 6: 2 shifts + 8 ANDs per word), the general kernel three copies
//    (<< 4, >> 2, >> 8: 3 shifts + 8 ANDs).  Products of
//    different j carry different power-of-two factors, so they go to three accumulators
//    that are combined once per tile: sum_j 2^(24-2j) acc_j = sum_k x_k c_k.  With
//    c = w + 1 the result is sum_k x_k c_k - sum_k x_k; the second sum comes from one more
//    group of MFMAs per wave whose 16-row operand is a constant, and seeds the accumulator.
//  * Split-K partial tiles of the NW waves are added in a fixed order through LDS, scaled
//    by gamma, rounded to fp16 (RNE) and stored.  No atomics: results are deterministic.
//  * One launch can carry up to 32 independent jobs (a job = one matrix and at most 16, in
//    one variant 32, activation rows); a workgroup finds its job from its index.
//  * Four forms.  The stream form (gemv_stream_kernel: K up to 8 slices per pass) gives a wave
//    one slice for the whole kernel and a workgroup a run of consecutive tiles of one job, so
//    activations are staged once and only weights move afterwards.  The lean form
//    (gemv_lean_kernel) is the stream form cut down to the decode shapes (one pass over K, one
//    block of 16 rows, one gamma, N a multiple of 16) and is what those launches run.  The
//    long-K form (gemv_longk_kernel) takes lone calls with 4096 < K <= 16384 whose workgroups
//    get one or two tiles each: a wave walks its up to four slices with the next one's data
//    already in flight.  The general form (gemv_kernel) loops a wave over slices and a
//    workgroup over items of any job; it takes the calls with K > 4096 that are too small
//    for the stream form's passes to pay and that the long-K form does not cover (K > 16384,
//    N not a multiple of 16, more than 512 tiles).
#include "tl_internal.hpp"
#include "tl_deal.hpp"

#include <cstddef>
#include <type_traits>

namespace tl {

namespace {

constexpr int kTMax = 4;          // tiles per work item
constexpr int kSliceK = 512;      // K elements a wave owns per pass
constexpr int kWaveLds = 16384;   // bytes of LDS per wave: 16 activation rows x 1 KB
constexpr int kMaxJobs = 32;      // jobs per launch (the table is 2.7 KB of kernel arguments)

struct GemvJob {                  // 80 bytes, lives in the kernel argument segment
    const __half* x;              // first activation row of this 16-row block
    const uint32_t* W;
    __half* y;                    // first output row of this block
    float gamma;
    int Mrem;                     // 1..16 activation rows (stream form with two row blocks: 1..32)
    int N, K;
    int tiles;                    // ceil(N / 16)
    int items;                    // general form: work items of this job, ceil(tiles / T)
    int slices;                   // ceil(K / 512)
    int mr;                       // general form: staged rows, the power of two >= Mrem
    int run, plus;                // stream form: tiles per workgroup, and how many of the job's first workgroups take one more
    const __half* scales;         // per-group scales [K / group][N] (kernels with GS), else unused
    int hpg;                      // per-group scales: scale units of a slice per group
    int reserved;
};

struct GemvBatch {
    int count;
    int total_items;
    int red_off;                  // byte offset in LDS of the split-K reduction area
    int pad;
    int item0[kMaxJobs];          // first work item of job j; INT_MAX for unused entries
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

// What a workgroup needs to know about one work item; every member is wave-uniform.
struct ItemCtx {
    const unsigned char* Wb;
    const unsigned char* xb;
    __half* y;
    float gamma;
    int Mrem, MR;
    int N, K;
    uint32_t row_bytes;           // bytes per packed row
    int chunks;                   // 64-weight (16-byte) chunks per row
    int tiles, items, idx;        // tile t of the item is idx + t * items
    int slices;
    const unsigned char* sc;      // per-group scales [K / group][N] fp16, and 256-weight halves per group
    int hpg;
};

// The job table of a launch, one job per lane (lanes 0 .. kMaxJobs - 1), read from the kernel argument
// segment with vector loads: every workgroup needs one entry chosen by its index, and a
// scalar look-up would be two dependent trips to memory before the first weight is requested.
struct JobTable {
    uint32_t d[20];               // the 20 dwords of GemvJob
    int item0;
};

__device__ __forceinline__ JobTable load_table(int lane)
{
    typedef const __attribute__((address_space(4))) unsigned char* kptr;
    kptr ka = (kptr)__builtin_amdgcn_kernarg_segment_ptr();     // GemvBatch is the only argument
    const int k = lane & (kMaxJobs - 1);
    JobTable r;
    r.item0 = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < 20; ++i) r.d[i] = 0u;
    // only lanes 0 .. kMaxJobs - 1 load (the entries are read with v_readlane from those lanes): half
    // of the addresses for the CU's address path, which all eight waves go through at once
    if (lane < kMaxJobs) {
        r.item0 = *(const __attribute__((address_space(4))) int*)(ka + offsetof(GemvBatch, item0) + 4 * k);
        const __attribute__((address_space(4))) u32x4* jp =
            (const __attribute__((address_space(4))) u32x4*)(ka + offsetof(GemvBatch, job) + sizeof(GemvJob) * k);
#pragma unroll
        for (int i = 0; i < 5; ++i) {
            const u32x4 q = jp[i];
            r.d[4 * i] = q[0]; r.d[4 * i + 1] = q[1]; r.d[4 * i + 2] = q[2]; r.d[4 * i + 3] = q[3];
        }
    }
    return r;
}

// Work item g -> its job (the last one whose first item is <= g) and position in it.
__device__ __forceinline__ ItemCtx load_item(const JobTable& tb, int g)
{
    const unsigned long long m = __builtin_amdgcn_ballot_w64(g >= tb.item0) & ((1ull << kMaxJobs) - 1);
    const int ji = __builtin_popcountll(m) - 1;
    uint32_t f[20];
#pragma unroll
    for (int i = 0; i < 19; ++i) f[i] = __builtin_amdgcn_readlane(tb.d[i], ji);
    const int item0 = __builtin_amdgcn_readlane(tb.item0, ji);
    ItemCtx c;
    c.xb = reinterpret_cast<const unsigned char*>(uintptr_t(f[0]) | (uintptr_t(f[1]) << 32));
    c.Wb = reinterpret_cast<const unsigned char*>(uintptr_t(f[2]) | (uintptr_t(f[3]) << 32));
    c.y = reinterpret_cast<__half*>(uintptr_t(f[4]) | (uintptr_t(f[5]) << 32));
    c.gamma = __builtin_bit_cast(float, f[6]);
    c.Mrem = int(f[7]);
    c.N = int(f[8]); c.K = int(f[9]);
    c.row_bytes = f[9] >> 2;
    c.chunks = int(f[9] >> 6);
    c.tiles = int(f[10]); c.items = int(f[11]); c.idx = g - item0;
    c.slices = int(f[12]);
    c.MR = int(f[13]);
    c.sc = reinterpret_cast<const unsigned char*>(uintptr_t(f[16]) | (uintptr_t(f[17]) << 32));
    c.hpg = int(f[18]);
    return c;
}

static_assert(sizeof(GemvJob) == 80 && offsetof(GemvJob, gamma) == 24 && offsetof(GemvJob, mr) == 52 &&
              offsetof(GemvJob, run) == 56 && offsetof(GemvJob, scales) == 64 && offsetof(GemvJob, hpg) == 72,
              "load_item decodes GemvJob by dword position");

// T: tiles per work item; MULTI: the launch carries more than one job.
// A workgroup takes the items blockIdx.x, blockIdx.x + gridDim.x, ...
template <int T, bool MULTI>
__global__ void __launch_bounds__(512)
gemv_kernel(GemvBatch b)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int NW = blockDim.x >> 6;
    unsigned char* const my_lds = lds_raw + wave * kWaveLds;

    // ---- coalesced load mapping: 8 lanes per 128-byte line, 8 rows per instruction ----
    const int lr = lane >> 3;                  // row within the half tile
    const int lc = lane & 7;                   // chunk within the slice
    // ---- MFMA mapping: lane (i, g) = (row / activation column, k group) -----------------
    const int mi = lane & 15;
    const int mg = lane >> 4;

    // LDS offsets (bytes, relative to my_lds); immediates add the row / tile / half part
    const uint32_t ww_off = uint32_t(lr) * 128u + (uint32_t(lc ^ lr) << 4);
    const uint32_t wr_off0 = uint32_t(mi) * 128u + (uint32_t((mg) ^ (mi & 7)) << 4);
    const uint32_t wr_off1 = uint32_t(mi) * 128u + (uint32_t((4 + mg) ^ (mi & 7)) << 4);

    u32x4 wreg[T][2];
    auto issue_w = [&](const ItemCtx& c, int t, int slice) {
        int tile = c.idx + t * c.items;
        if (tile >= c.tiles) tile = c.tiles - 1;           // loaded again, never used
        int chunk = slice * 8 + lc;
        if (chunk >= c.chunks) chunk = 0;                  // multiplied by zero activations
        const unsigned char* tb = c.Wb + size_t(tile) * 16u * c.row_bytes;
        uint32_t off0 = uint32_t(lr) * c.row_bytes + uint32_t(chunk) * 16u;
        uint32_t off1 = off0 + 8u * c.row_bytes;
        if ((c.N & 15) != 0 && tile == c.tiles - 1) {      // scalar branch: rows past N read row N-1
            const int last = c.N - 1 - tile * 16;
            off0 = uint32_t(lr < last ? lr : last) * c.row_bytes + uint32_t(chunk) * 16u;
            off1 = uint32_t(lr + 8 < last ? lr + 8 : last) * c.row_bytes + uint32_t(chunk) * 16u;
        }
        // the pointers were put together from table registers: say that they are global
        typedef const __attribute__((address_space(1))) u32x4* gptr;
        wreg[t][0] = __builtin_nontemporal_load((gptr)(tb + off0));
        wreg[t][1] = __builtin_nontemporal_load((gptr)(tb + off1));
    };

    // Activation rows go straight from global memory into the LDS staging area (LDS-DMA, no
    // registers): one instruction per staged row, lane l fetches the 16-byte piece
    // l ^ (r & 7) of the slice and the hardware drops it at slot l, which is the swizzled
    // layout the operand set-up reads.  Rows past Mrem repeat row Mrem-1; lanes past K
    // store zeros instead (their weights are whatever chunk 0 holds).
    auto issue_x = [&](const ItemCtx& c, int slice) {
        for (int r = 0; r < c.MR; ++r) {
            const int rr = r < c.Mrem ? r : c.Mrem - 1;
            const int kx = slice * kSliceK + ((lane ^ (r & 7)) << 3);
            if (kx < c.K) {
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)(c.xb + size_t(rr) * c.K * 2 + uint32_t(kx) * 2u),
                    (__attribute__((address_space(3))) void*)(my_lds + r * 1024),
                    16, 0, 0);
            } else {
                *reinterpret_cast<u32x4*>(my_lds + r * 1024 + (uint32_t(lane) << 4)) = u32x4{0u, 0u, 0u, 0u};
            }
        }
    };

    // One pass of a wave: 512 k of the T tiles of an item.  FIRST (a compile-time tag) marks
    // the very first pass of the workgroup, whose activations were requested before its
    // weights; that copy of the body runs straight from the kernel entry, so the compiler's
    // wait counts in it are exact and tile t is decoded as soon as its own two loads have
    // arrived.  Every other pass starts with all of its loads complete.
    auto do_pass = [&](auto first_tag, const ItemCtx& cur, const ItemCtx& nxt, bool pre, int slice,
                       f32x4 (&part)[T]) {
        constexpr bool FIRST = decltype(first_tag)::value;
        // The compiler does not track LDS-DMA, so wait by hand.  First pass: until only the
        // 2T weight loads issued after the activation rows are outstanding (loads of a wave
        // return in order).  Later passes: weights were requested first, so for all.
        if constexpr (FIRST) __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * T));
        else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        const bool more = (slice + NW) < cur.slices;

        const int xrow = mi & (cur.MR - 1);                // staged activation row of this lane's column
        const uint32_t xr_off = uint32_t(xrow) * 1024u + uint32_t(mg) * 128u;
        const uint32_t sw = uint32_t(xrow & 7);
        // ---------------- activations of this slice -> MFMA B registers --------------------
        // staging layout: row r, 16-byte piece P at slot P ^ (r & 7)
        // breg[h][wd][e]: (x[k], x[k + 8]) with k = slice0 + 64 (4h + g) + 16 wd + e
        uint32_t breg[2][4][8];
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
        // ---------------- per tile: turn through LDS, decode, MFMA ---------------------------
        // The staging rows are dead once breg is built, so region t (2 KB) reuses them; LDS
        // operations of one wave execute in order.
#pragma unroll
        for (int t = 0; t < T; ++t) {
            unsigned char* const reg_t = my_lds + t * 2048;
            *reinterpret_cast<u32x4*>(reg_t + ww_off) = wreg[t][0];
            *reinterpret_cast<u32x4*>(reg_t + 1024 + ww_off) = wreg[t][1];
            if (more) issue_w(cur, t, slice + NW);         // refill for the next pass
            else if (pre) issue_w(nxt, t, wave);           // or for the next item
            if (cur.idx + t * cur.items < cur.tiles) {     // scalar: tiles past the end are skipped
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
        }
        // The staging rows share LDS with the tile regions, so the next activations can only
        // be fetched once the last tile has been read; the next pass waits for them.
        if (more) issue_x(cur, slice + NW);
        else if (pre) issue_x(nxt, wave);
    };

    // Split-K reduction across the waves and output.  Layout [t][wave][lane] of f32x4 in LDS.
    // A workgroup with a single item reuses the staging space (red_off = 0); otherwise the
    // area lies behind it, because the next item's activations are already arriving there.
    // The first barrier also keeps this item's partial sums from overtaking a wave that
    // still reads the previous ones.
    // The barriers wait for LDS traffic only (s_waitcnt lgkmcnt(0); s_barrier): the next item's
    // weights and activations stay in flight across them, which __syncthreads would drain.
    auto lds_barrier = [&]() {
        __builtin_amdgcn_s_waitcnt(0xF | (0x3 << 14) | (0x7 << 4));
        __builtin_amdgcn_s_barrier();
    };
    auto epilogue = [&](const ItemCtx& cur, const f32x4 (&part)[T]) {
        lds_barrier();
        f32x4* red = reinterpret_cast<f32x4*>(lds_raw + b.red_off);
#pragma unroll
        for (int t = 0; t < T; ++t) red[(t * NW + wave) * 64 + lane] = part[t];
        lds_barrier();
        const float gamma = cur.gamma;
        for (int o = threadIdx.x; o < T * 64; o += blockDim.x) {
            const int t = o >> 6;
            const int l = o & 63;
            const int tile = cur.idx + t * cur.items;
            if (tile >= cur.tiles) continue;
            f32x4 v[8];
#pragma unroll
            for (int w = 0; w < 8; ++w)                     // all reads in flight, then a fixed-order sum
                v[w] = (w < NW) ? red[(t * NW + w) * 64 + l] : f32x4{0.f, 0.f, 0.f, 0.f};
            const f32x4 s = ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
            const int n = tile * 16 + 4 * (l >> 4);
            if ((l & 15) < cur.Mrem) {
                typedef __attribute__((address_space(1))) __half* gh_ptr;
                gh_ptr dst = (gh_ptr)(cur.y + size_t(l & 15) * cur.N + n);
                if (n + 3 < cur.N && (cur.N & 3) == 0) {    // four consecutive n: one 8-byte store
                    const f16x2 lo = {(_Float16)(gamma * s[0]), (_Float16)(gamma * s[1])};
                    const f16x2 hi = {(_Float16)(gamma * s[2]), (_Float16)(gamma * s[3])};
                    *(__attribute__((address_space(1))) u32x2*)dst =
                        u32x2{__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (n + r < cur.N) *(__attribute__((address_space(1))) _Float16*)(dst + r) = (_Float16)(gamma * s[r]);
                }
            }
        }
    };

    int g = blockIdx.x;
    // A launch of one job reads it with scalar loads at fixed offsets (one trip to memory,
    // nothing depends on a look-up); several jobs go through the table in registers.
    JobTable table;
    if constexpr (MULTI) table = load_table(lane);
    auto get_item = [&](int gi) -> ItemCtx {
        if constexpr (MULTI) {
            return load_item(table, gi);
        } else {
            const GemvJob& J = b.job[0];
            ItemCtx c;
            c.xb = reinterpret_cast<const unsigned char*>(J.x);
            c.Wb = reinterpret_cast<const unsigned char*>(J.W);
            c.y = J.y;
            c.gamma = J.gamma;
            c.Mrem = J.Mrem; c.MR = J.mr;
            c.N = J.N; c.K = J.K;
            c.row_bytes = uint32_t(J.K) >> 2;
            c.chunks = J.K >> 6;
            c.tiles = J.tiles; c.items = J.items; c.idx = gi;
            c.slices = J.slices;
            return c;
        }
    };
    ItemCtx cur = get_item(g);
    // Activations go first: they are short L2 hits, and the loads of one wave return in
    // order, so the weight stream queued behind them overlaps the operand set-up.
    if (wave < cur.slices) {
        issue_x(cur, wave);
#pragma unroll
        for (int t = 0; t < T; ++t) issue_w(cur, t, wave);
    }
    // The next item of this workgroup: its first weights and activations are requested
    // during the last pass over the current one, so HBM stays busy through the epilogue.
    int gn = g + int(gridDim.x);
    bool has_next = gn < b.total_items;
    ItemCtx nxt = get_item(has_next ? gn : g);
    bool pre = has_next && wave < nxt.slices;

    f32x4 part[T];
#pragma unroll
    for (int t = 0; t < T; ++t) part[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    int slice = wave;
    if (slice < cur.slices) {
        do_pass(std::true_type{}, cur, nxt, pre, slice, part);
        slice += NW;
    }
    for (;;) {
        for (; slice < cur.slices; slice += NW)             // wave-uniform trip count
            do_pass(std::false_type{}, cur, nxt, pre, slice, part);
        if (wave >= cur.slices && pre) {                    // a wave with no slice of this item
            issue_x(nxt, wave);
#pragma unroll
            for (int t = 0; t < T; ++t) issue_w(nxt, t, wave);
        }
        epilogue(cur, part);
        if (!has_next) break;
        cur = nxt;
        g = gn;
        gn = g + int(gridDim.x);
        has_next = gn < b.total_items;
        nxt = get_item(has_next ? gn : g);
        pre = has_next && wave < nxt.slices;
#pragma unroll
        for (int t = 0; t < T; ++t) part[t] = f32x4{0.f, 0.f, 0.f, 0.f};
        slice = wave;
    }
}

// LDS per wave of the stream form: 16 KB of activation staging, or two tile regions and two
// sets of T partial-sum tiles, whichever is more.
constexpr int stream_wave_lds(int T)
{
    return 4096 + 2 * T * 1024 > kWaveLds ? 4096 + 2 * T * 1024 : kWaveLds;
}

// ------------------------------------------------------------------------------------------
// Stream form of the kernel, for launches in which every job has K <= 512 * (waves per group):
// wave w owns K slice w for good, so its activations are fetched and turned into MFMA operands
// once, and all that moves afterwards is the weight stream.  A workgroup serves one job (its
// index picks the job; GemvBatch::item0[j] is the first workgroup of job j) and walks a run of
// consecutive tiles of it, T at a time (GemvJob::run, plus: tiles per workgroup, and how many of the
// job's first workgroups take one more).  While item i is decoded the loads of item i + 1 are in flight,
// each tile waits only for its own two loads, and there is one LDS-only barrier per item.
// The loop body holds nothing but weight loads and the output stores, which is what keeps the
// compiler's wait counts exact; the last item is a second copy of the body without refills.
// PASSES: some job of the launch has K longer than the waves' slices together.
// NB: blocks of 16 activation rows a job may have (1 or 2).  With two, every decoded weight
// operand feeds two MFMAs, one per block: the decode, which is what limits the kernel, is paid
// once for 32 rows.  With PASSES the kept sums take 1 KB per tile and row block.
// GS: per-group scales (Sec. 3.3, CPU inference: one fp16 scale per block along K; App. on the
// GPU kernel: scales kept in a separate buffer) instead of one gamma: the GS (2 or 4) scale units
// of a slice, 256 or 128 weights each, are accumulated apart, each multiplied by the scale of its
// group and output row.  Groups are multiples of 128 weights; the scales lie as [K / group][N].
template <int T, bool MULTI, bool PASSES, int NB, int GS = 0>
__global__ void __launch_bounds__(512)
gemv_stream_kernel(GemvBatch b)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int NW = blockDim.x >> 6;
    // LDS of a wave: activation rows (16 KB) while the operands are built; afterwards two tile
    // regions at 0 and 2 KB, and from 4 KB two sets of T NB partial-sum tiles (1 KB each).
    // GS: 0, or the number of scale units in a wave's 512-weight slice: 2 (units of 256 weights, an
    // MFMA's whole k range) or 4 (units of 128: an MFMA's lane groups 0,1 and 2,3 lie in different
    // units, so every product is issued twice, each time with the other pair's weights masked off)
    static_assert(GS == 0 || ((GS == 2 || GS == 4) && NB == 1 && MULTI), "per-group scales: one row block, job table");
    constexpr int H = GS ? GS : 1;            // accumulator sets per tile: one per scale unit
    constexpr int kStride = stream_wave_lds(T * NB);
    unsigned char* const my_lds = lds_raw + wave * kStride;

    const int lr = lane >> 3, lc = lane & 7;   // load mapping: row of the half tile, chunk of the slice
    const int mi = lane & 15, mg = lane >> 4;  // MFMA mapping: row / activation column, k group
    const uint32_t ww_off = uint32_t(lr) * 128u + (uint32_t(lc ^ lr) << 4);
    const uint32_t wr_off0 = uint32_t(mi) * 128u + (uint32_t((mg) ^ (mi & 7)) << 4);
    const uint32_t wr_off1 = uint32_t(mi) * 128u + (uint32_t((4 + mg) ^ (mi & 7)) << 4);

    // ---- this workgroup's job and run of items ----------------------------------------------
    ItemCtx J;
    int ipg, plus;
    if constexpr (MULTI) {
        const JobTable table = load_table(lane);
        J = load_item(table, int(blockIdx.x));             // idx: position among the job's workgroups
        const unsigned long long m = __builtin_amdgcn_ballot_w64(int(blockIdx.x) >= table.item0) & ((1ull << kMaxJobs) - 1);
        const int ji = __builtin_popcountll(m) - 1;
        ipg = int(__builtin_amdgcn_readlane(table.d[14], ji));
        plus = int(__builtin_amdgcn_readlane(table.d[15], ji));
    } else {
        const GemvJob& G = b.job[0];
        J.xb = reinterpret_cast<const unsigned char*>(G.x);
        J.Wb = reinterpret_cast<const unsigned char*>(G.W);
        J.y = G.y;
        J.gamma = G.gamma;
        J.Mrem = G.Mrem; J.MR = G.mr;
        J.N = G.N; J.K = G.K;
        J.row_bytes = uint32_t(G.K) >> 2;
        J.chunks = G.K >> 6;
        J.tiles = G.tiles; J.items = G.items; J.idx = int(blockIdx.x);
        J.slices = G.slices;
        ipg = G.run; plus = G.plus;
    }
    const int local = J.idx;
    const int tile0 = local * ipg + (local < plus ? local : plus);      // first tile of the run
    const int tile_end = tile0 + ipg + (local < plus ? 1 : 0);
    const int n_items = (tile_end - tile0 + T - 1) / T;
    // K longer than the waves' slices together (NW x 512) is walked in passes: pass c gives wave
    // w the slice c NW + w, streams the whole run of tiles, and leaves the sums of the run in
    // LDS (1 KB per tile behind the waves' areas) for the next pass to add to.
    const int n_pass = PASSES ? (J.slices + NW - 1) / NW : 1;
    unsigned char* const ysum = lds_raw + NW * kStride;
    int slice = wave;
    bool active = slice < J.slices;
    uint32_t col_off = 0;
    const bool ragged_n = (J.N & 15) != 0;
    typedef const __attribute__((address_space(1))) u32x4* gptr;

    u32x4 wreg[T][2];
    f16x4 sreg[T][H];                          // GS: the scales of the lane's four output rows, per unit
    uint32_t sc_off[H] = {};                   // GS: byte offset of the units' groups in the scales
    // GS == 4: all ones in the lanes whose k lies in the first (second) unit of an MFMA's range
    const uint32_t pair_mask[2] = {(lane >> 5) == 0 ? 0xFFFFFFFFu : 0u, (lane >> 5) == 1 ? 0xFFFFFFFFu : 0u};
    auto chunk_offset = [&](int sl) {
        int chunk = sl * 8 + lc;                           // 16-byte chunk of this lane within the row
        if (chunk >= J.chunks) chunk = 0;                  // past K: multiplied by zero activations
        return uint32_t(chunk) * 16u;
    };
    // Several passes, one row block of at most 4 rows: the next pass's activation rows are fetched
    // into registers while the last item of this pass is worked on (plain loads, so the compiler's
    // wait counts stay exact), and that item refills with the next pass's first weights.
    constexpr bool kAheadOk = PASSES && NB == 1 && GS == 0;
    u32x4 xpre[kAheadOk ? 4 : 1];
    auto issue_w = [&](int first, int t) {
        int tile = first + t;
        if (tile >= tile_end) tile = tile_end - 1;         // past the run: its last tile again, never stored
        const unsigned char* tb = J.Wb + size_t(tile) * 16u * J.row_bytes;
        // rows past N read row N-1 (no branch: the loop body stays one scheduling region)
        const int last = (ragged_n && tile == J.tiles - 1) ? J.N - 1 - tile * 16 : 15;
        const uint32_t off0 = uint32_t(lr < last ? lr : last) * J.row_bytes + col_off;
        const uint32_t off1 = uint32_t(lr + 8 < last ? lr + 8 : last) * J.row_bytes + col_off;
        wreg[t][0] = __builtin_nontemporal_load((gptr)(tb + off0));
        wreg[t][1] = __builtin_nontemporal_load((gptr)(tb + off1));
        if constexpr (GS) {
            int n0 = tile * 16 + 4 * mg;                   // the lane's rows of the result: n0 .. n0 + 3
            if (n0 > J.N - 4) n0 = J.N - 4;                // rows past N (N % 4 == 0): any scale will do
#pragma unroll
            for (int hh = 0; hh < H; ++hh)
                sreg[t][hh] = *(const __attribute__((address_space(1))) f16x4*)(J.sc + sc_off[hh] + uint32_t(n0) * 2u);
        }
    };

    uint32_t breg[NB][2][4][8];                // this wave's activations as MFMA B operands, per row block
    f32x4 nsx[NB][H];                          // -2^-20 sum_k x[m][k] over the slice (GS: each half), as an accumulator
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int hh = 0; hh < H; ++hh) nsx[nb][hh] = f32x4{0.f, 0.f, 0.f, 0.f};
    // Start of a pass: fetch this wave's activation slice and the first item's weights together,
    // then turn the activations into operand registers.
    // ahead_here: the end of the pass before has requested this pass's activation rows (into xpre)
    // and its first item's weights already.
    auto begin_pass = [&](int pass, bool ahead_here) {
    slice = pass * NW + wave;
    active = slice < J.slices;
    if (!ahead_here) col_off = chunk_offset(slice);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int hh = 0; hh < H; ++hh) nsx[nb][hh] = f32x4{0.f, 0.f, 0.f, 0.f};
    if constexpr (GS) {
        // groups of this wave's units (J.hpg units per group); a unit past K (its activations are
        // zeros) takes the last group
        const int last_group = (J.K - 1) / ((kSliceK / H) * J.hpg);
#pragma unroll
        for (int hh = 0; hh < H; ++hh) {
            int g = (H * slice + hh) / J.hpg;
            if (g > last_group) g = last_group;
            sc_off[hh] = uint32_t(g) * uint32_t(J.N) * 2u;
        }
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        // rows of this block: block 0 takes the first 16 (or fewer), block 1 what is left
        const int rows = nb == 0 ? (J.Mrem < 16 ? J.Mrem : 16) : J.Mrem - 16;
        int mr = 1;
        while (mr < rows) mr *= 2;
        if (active && rows > 0) {
            // activation rows by LDS-DMA, swizzled: lane l fetches piece l ^ (r & 7) of row r.
            // Kept as short rolled loops: this is on the way to the first weight load, and at
            // the start of a kernel every instruction line is a miss in the instruction cache.
            // Staged rows past `rows` are never written: an MFMA column depends on its own column
            // of B alone, and the outputs of those columns are not stored.
            typedef const __attribute__((address_space(1))) unsigned char* gbytes;
            const size_t row_stride = size_t(J.K) * 2;
            gbytes src = (gbytes)(J.xb + size_t(16 * nb) * row_stride + size_t(slice) * (kSliceK * 2));
            if (kAheadOk && ahead_here) {
                if constexpr (kAheadOk) {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (r < rows) *reinterpret_cast<u32x4*>(my_lds + r * 1024 + (uint32_t(lane) << 4)) = xpre[r];
                }
            } else if ((slice + 1) * kSliceK <= J.K) {     // the whole slice lies inside K
                const uint32_t lane16 = uint32_t(lane) << 4;
#pragma unroll 1
                for (int r = 0; r < rows; ++r) {
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + (lane16 ^ (uint32_t(r & 7) << 4))),
                                                     (__attribute__((address_space(3))) void*)(my_lds + r * 1024), 16, 0, 0);
                    src += row_stride;
                }
            } else {
#pragma unroll 1
                for (int r = 0; r < rows; ++r) {
                    const int kk = (lane ^ (r & 7)) << 3;  // first of this lane's 8 activations within the slice
                    if (slice * kSliceK + kk < J.K) {
                        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + uint32_t(kk) * 2u),
                                                         (__attribute__((address_space(3))) void*)(my_lds + r * 1024), 16, 0, 0);
                    } else {
                        *reinterpret_cast<u32x4*>(my_lds + r * 1024 + (uint32_t(lane) << 4)) = u32x4{0u, 0u, 0u, 0u};
                    }
                    src += row_stride;
                }
            }
            if (kAheadOk && ahead_here) {
                // nothing to request; the registers' own loads are waited for by the compiler
            } else if (nb == 0) {
#pragma unroll
                for (int t = 0; t < T; ++t) issue_w(tile0, t);
                // the compiler does not track LDS-DMA: wait until only the 2T weight loads are outstanding
                __builtin_amdgcn_s_waitcnt(vmcnt_imm((2 + GS) * T));
            } else {
                __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // requested after the weights: wait for all
            }
            const int xrow = mi & (mr - 1);
            const uint32_t xr_off = uint32_t(xrow) * 1024u + uint32_t(mg) * 128u;
            const uint32_t sw = uint32_t(xrow & 7);
            // breg[nb][h][wd][e]: (x[k], x[k + 8]) with k = slice0 + 64 (4h + g) + 16 wd + e.
            // Columns that stand for no activation row get zeros (byte selector 0x0c), not the
            // unwritten staging rows: nothing is stored from them, and multiplying zeros costs
            // the matrix pipes less power than multiplying copies of real rows.
            const bool live = mi < rows;
            const uint32_t sel_lo = live ? 0x05040100u : 0x0c0c0c0cu;
            const uint32_t sel_hi = live ? 0x07060302u : 0x0c0c0c0cu;
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
                        breg[nb][h][wd][2 * r] = __builtin_amdgcn_perm(hi[r], lo[r], sel_lo);
                        breg[nb][h][wd][2 * r + 1] = __builtin_amdgcn_perm(hi[r], lo[r], sel_hi);
                    }
                }
            const uint32_t c = 0x80108010u;               // fp16 pair of -2^-20
            const u32x4 a = u32x4{c, c, c, c};
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const u32x4 bb = u32x4{breg[nb][h][0][e], breg[nb][h][1][e], breg[nb][h][2][e], breg[nb][h][3][e]};
                    if constexpr (GS == 4) {
#pragma unroll
                        for (int q = 0; q < 2; ++q) {
                            const u32x4 aq = a & pair_mask[q];
                            nsx[nb][2 * h + q] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(aq), as_f16x8(bb), nsx[nb][2 * h + q], 0, 0, 0);
                        }
                    } else {
                        nsx[nb][GS ? h : 0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(a), as_f16x8(bb), nsx[nb][GS ? h : 0], 0, 0, 0);
                    }
                }
            if (NB > 1 && nb == 0) __builtin_amdgcn_s_waitcnt(0xF | (0x3 << 14) | (0x7 << 4));   // staging read before it is refilled
        } else {
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int wd = 0; wd < 4; ++wd)
#pragma unroll
                    for (int e = 0; e < 8; ++e) breg[nb][h][wd][e] = 0u;
        }
    }
    };

    // One item (tiles first .. first + T - 1): tile t goes through LDS region t & 1 into MFMA
    // order, is decoded and multiplied; REFILL: its registers are loaded again at once for the
    // next item.  Tiles past the run are computed from whatever was loaded and never stored.
    auto item = [&](auto refill_tag, int first, int refill_first, int parity, bool first_pass_rt, bool last_pass_rt) {
        constexpr bool REFILL = decltype(refill_tag)::value;
        const bool first_pass = PASSES ? first_pass_rt : true;
        const bool last_pass = PASSES ? last_pass_rt : true;
        f32x4 part[NB][T];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int t = 0; t < T; ++t) part[nb][t] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (active) {
#pragma unroll
            for (int t = 0; t < T; ++t) {
                unsigned char* const reg_t = my_lds + (t & 1) * 2048;
                *reinterpret_cast<u32x4*>(reg_t + ww_off) = wreg[t][0];
                *reinterpret_cast<u32x4*>(reg_t + 1024 + ww_off) = wreg[t][1];
                f16x4 sc_cur[H];                           // this tile's scales, before the refill replaces them
#pragma unroll
                for (int hh = 0; hh < H; ++hh) sc_cur[hh] = sreg[t][hh];
                if constexpr (REFILL) issue_w(refill_first, t);
                if (REFILL || first + t < tile_end) {      // the last item may be short
                    f32x4 acc[NB][H][3];
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                        for (int hh = 0; hh < H; ++hh) {
                            acc[nb][hh][0] = nsx[nb][hh];
                            acc[nb][hh][1] = f32x4{0.f, 0.f, 0.f, 0.f};
                            acc[nb][hh][2] = f32x4{0.f, 0.f, 0.f, 0.f};
                        }
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const u32x4 wv = *reinterpret_cast<const u32x4*>(reg_t + (h ? wr_off1 : wr_off0));
                        // element e of each half-word sits at bits 2e, 2e+1; the mantissa bits
                        // 4..9 (classes 0..2 -> accumulators) hold e = 2,3,4 as loaded, e = 0,1
                        // after << 4 and e = 5,6,7 after >> 6
                        const u32x4 sh[3] = {wv << 4, wv, wv >> 6};
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const int src = e < 2 ? 0 : (e < 5 ? 1 : 2);
                            const int j = e < 2 ? e : (e < 5 ? e - 2 : e - 5);
                            const uint32_t mask = 0x00300030u << (2 * j);
                            const u32x4 a = sh[src] & mask;
#pragma unroll
                            for (int nb = 0; nb < NB; ++nb) {
                                const u32x4 bb = u32x4{breg[nb][h][0][e], breg[nb][h][1][e], breg[nb][h][2][e], breg[nb][h][3][e]};
                                if constexpr (GS == 4) {
#pragma unroll
                                    for (int q = 0; q < 2; ++q) {
                                        const u32x4 aq = sh[src] & (mask & pair_mask[q]);
                                        acc[nb][2 * h + q][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(aq), as_f16x8(bb), acc[nb][2 * h + q][j], 0, 0, 0);
                                    }
                                } else {
                                    acc[nb][GS ? h : 0][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(a), as_f16x8(bb), acc[nb][GS ? h : 0][j], 0, 0, 0);
                                }
                            }
                        }
                    }
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        if constexpr (GS) {
                            // register r of the accumulator is output row 4 (lane / 16) + r of the tile
                            f32x4 sum = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                            for (int hh = 0; hh < H; ++hh) {
                                const f32x4 sc = f32x4{float(sc_cur[hh][0]), float(sc_cur[hh][1]), float(sc_cur[hh][2]), float(sc_cur[hh][3])};
                                sum += sc * (acc[nb][hh][0] * 1048576.f + acc[nb][hh][1] * 262144.f + acc[nb][hh][2] * 65536.f);
                            }
                            part[nb][t] = sum;
                        } else {
                            part[nb][t] = acc[nb][0][0] * 1048576.f + acc[nb][0][1] * 262144.f + acc[nb][0][2] * 65536.f;
                        }
                    }
                }
            }
        }
        // split-K: partial sums into this wave's set `parity`, one barrier, fixed-order sum.
        // The other set is still being read by waves that lag one item behind, never more:
        // they must pass this item's barrier before anybody writes that set again.
        unsigned char* const red = my_lds + 4096 + parity * (T * NB * 1024);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int t = 0; t < T; ++t) reinterpret_cast<f32x4*>(red + (nb * T + t) * 1024)[lane] = part[nb][t];
        __builtin_amdgcn_s_waitcnt(0xF | (0x3 << 14) | (0x7 << 4));     // lgkmcnt(0): LDS only, loads stay in flight
        __builtin_amdgcn_s_barrier();
        if (const int o = threadIdx.x; o < T * NB * 64) {  // T NB <= waves: one output quad per thread
            const int q = o >> 6;                           // nb * T + t
            const int nb = q / T;
            const int t = q - nb * T;
            const int l = o & 63;
            const int row = 16 * nb + (l & 15);
            const int tile = first + t;
            f32x4 v[8];
#pragma unroll
            for (int w = 0; w < 8; ++w)
                v[w] = (w < NW) ? reinterpret_cast<const f32x4*>(lds_raw + w * kStride + 4096 + parity * (T * NB * 1024) + q * 1024)[l]
                                : f32x4{0.f, 0.f, 0.f, 0.f};
            f32x4 s = ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
            // sums of the earlier passes over K: kept by the thread that owns this output quad
            f32x4* const keep = reinterpret_cast<f32x4*>(ysum + ((tile - tile0) * NB + nb) * 1024) + l;
            if (!first_pass && tile < tile_end) s += *keep;
            if (!last_pass && tile < tile_end) *keep = s;
            const int n = tile * 16 + 4 * (l >> 4);
            if (last_pass && tile < tile_end && row < J.Mrem) {
                typedef __attribute__((address_space(1))) __half* gh_ptr;
                gh_ptr dst = (gh_ptr)(J.y + size_t(row) * J.N + n);
                const float gamma = GS ? 1.f : J.gamma;
                if (n + 3 < J.N && (J.N & 3) == 0) {       // four consecutive n: one 8-byte store
                    const f16x2 lo = {(_Float16)(gamma * s[0]), (_Float16)(gamma * s[1])};
                    const f16x2 hi = {(_Float16)(gamma * s[2]), (_Float16)(gamma * s[3])};
                    *(__attribute__((address_space(1))) u32x2*)dst =
                        u32x2{__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (n + r < J.N) *(__attribute__((address_space(1))) _Float16*)(dst + r) = (_Float16)(gamma * s[r]);
                }
            }
        }
    };

    bool ahead_here = false;
    for (int pass = 0; pass < n_pass; ++pass) {
        const bool first_pass = pass == 0, last_pass = pass + 1 == n_pass;
        begin_pass(PASSES ? pass : 0, ahead_here);
        ahead_here = false;
        int i = 0;
        for (; i + 1 < n_items; ++i) item(std::true_type{}, tile0 + i * T, tile0 + (i + 1) * T, i & 1, first_pass, last_pass);
        bool cross = false;
        if constexpr (kAheadOk) {
            const int next_slice = (pass + 1) * NW + wave;
            cross = !last_pass && active && next_slice < J.slices && J.Mrem <= 4;
            if (cross) {
                typedef const __attribute__((address_space(1))) unsigned char* gbytes;
                gbytes src = (gbytes)(J.xb + size_t(next_slice) * (kSliceK * 2));
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int piece = lane ^ (r & 7);      // the staging order of begin_pass
                    xpre[r] = u32x4{0u, 0u, 0u, 0u};
                    if (r < J.Mrem && next_slice * kSliceK + piece * 8 < J.K)
                        xpre[r] = *(gptr)(src + size_t(r) * (size_t(J.K) * 2) + uint32_t(piece) * 16u);
                }
                col_off = chunk_offset(next_slice);
                item(std::true_type{}, tile0 + i * T, tile0, i & 1, first_pass, last_pass);
                ahead_here = true;
            }
        }
        if (!cross) item(std::false_type{}, tile0 + i * T, 0, i & 1, first_pass, last_pass);
        if (PASSES && !last_pass) {
            // the next pass stages activations over the partial-sum sets: everybody must be done reading
            __builtin_amdgcn_s_waitcnt(0xF | (0x3 << 14) | (0x7 << 4));
            __builtin_amdgcn_s_barrier();
        }
    }
}

// ------------------------------------------------------------------------------------------
// Lean stream kernel: the stream form for launches in which every job takes one pass over K with
// the same number of 512-weight slices (= waves per workgroup), one block of at most 16
// activation rows, one gamma, and N a multiple of 16 -- the decode shapes.  What differs from
// gemv_stream_kernel is the way in and the loop, not the arithmetic:
//  * Every workgroup has a 64-byte record of its own in the kernel arguments (pointers of its job,
//    first tile and length of its run), read with one scalar load at an address that depends on
//    the workgroup index alone: no table search stands between the kernel entry and the first
//    requests, and one- and many-job launches run the same code.
//  * A lane's two weight addresses within a tile are computed once; a tile's loads are that
//    offset on a scalar base which steps from tile to tile, so the loop spends no vector
//    instructions on addresses.
//  * Every wave is active in every tile (no predicated tile bodies); the last item comes in one
//    copy per tile count.
// The vector ALU is what limits the steady state of these kernels (64 ANDs + 16 shifts + 16 MFMA
// issues + 8 combine operations per wave and tile are 104 of the ~120 issue slots a tile may
// take if the loop is to keep up with HBM), so every instruction that is not decode counts.
constexpr int kLeanMaxGroups = 256;

struct WgRec {                    // 64 bytes; rec[blockIdx.x] is read with scalar loads
    const unsigned char* W;       // packed row 0 of the first tile of the run
    const unsigned char* x;       // activations of the job, fp16 [Mrem][K]
    __half* y;                    // outputs of the job, fp16 [Mrem][N]
    float gamma;
    int K, N;
    int Mrem;                     // 1..16
    int tile0, ntiles;            // the run: tiles tile0 .. tile0 + ntiles - 1 of the job (ntiles >= 1)
    int pad[4];
};
static_assert(sizeof(WgRec) == 64, "one record per 64-byte line");

struct LeanBatch {
    WgRec rec[kLeanMaxGroups];
};

template <int T>
__global__ void __launch_bounds__(512)
gemv_lean_kernel(LeanBatch b)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int NW = blockDim.x >> 6;
    constexpr int kStride = stream_wave_lds(T);
    unsigned char* const my_lds = lds_raw + wave * kStride;
    typedef const __attribute__((address_space(1))) unsigned char* gbytes;

    const WgRec& R = b.rec[blockIdx.x];
    const int K = R.K, N = R.N, rows = R.Mrem, ntiles = R.ntiles;
    const unsigned char* const Wrun = R.W;
    const uint32_t row_bytes = uint32_t(K) >> 2;
    const uint32_t tile_bytes = 16u * row_bytes;

    const int lr = lane >> 3, lc = lane & 7;   // load mapping: row of the half tile, chunk of the slice
    const int mi = lane & 15, mg = lane >> 4;  // MFMA mapping: row / activation column, k group

    // ---- activations of this wave's slice: LDS-DMA, swizzled (lane l fetches piece l ^ (r & 7) of row r)
    {
        const size_t row_stride = size_t(K) * 2;
        gbytes src = (gbytes)(R.x + size_t(wave) * (kSliceK * 2));
        if ((wave + 1) * kSliceK <= K) {                    // the whole slice lies inside K
            const uint32_t lane16 = uint32_t(lane) << 4;
#pragma unroll 1
            for (int r = 0; r < rows; ++r) {
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + (lane16 ^ (uint32_t(r & 7) << 4))),
                                                 (__attribute__((address_space(3))) void*)(my_lds + r * 1024), 16, 0, 0);
                src += row_stride;
            }
        } else {
#pragma unroll 1
            for (int r = 0; r < rows; ++r) {
                const int kk = (lane ^ (r & 7)) << 3;      // first of this lane's 8 activations within the slice
                if (wave * kSliceK + kk < K) {
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + uint32_t(kk) * 2u),
                                                     (__attribute__((address_space(3))) void*)(my_lds + r * 1024), 16, 0, 0);
                } else {
                    *reinterpret_cast<u32x4*>(my_lds + r * 1024 + (uint32_t(lane) << 4)) = u32x4{0u, 0u, 0u, 0u};
                }
                src += row_stride;
            }
        }
    }
    // ---- weights: the lane's two 16-byte pieces of a tile, relative to the tile's first row
    uint32_t chunk = uint32_t(wave) * 8u + uint32_t(lc);
    if (chunk >= (uint32_t(K) >> 6)) chunk = 0;            // past K: multiplied by zero activations
    const uint32_t voff0 = uint32_t(lr) * row_bytes + chunk * 16u;
    const uint32_t voff1 = voff0 + 8u * row_bytes;
    // the run as a raw buffer (no stride, byte offsets, size = the run): base in scalar registers
    const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(Wrun), 0, uint32_t(ntiles) * tile_bytes, 0x00020000);
    u32x4 wreg[T][2];
    auto issue_w = [&](int idx, int t) {                   // idx: tile of the run; past the run: its last tile again
        const int c = idx < ntiles ? idx : ntiles - 1;
        // Buffer loads: descriptor and tile offset are scalar, the lane offset is a register that
        // never changes, so a request costs the vector ALU nothing.  That matters beyond the
        // instruction count: a wave whose data has arrived must get its next request out while
        // the other wave of its SIMD keeps the vector ALU busy.
        const uint32_t so = uint32_t(c) * tile_bytes;
        wreg[t][0] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(wres, voff0, so, 2));   // 2: nt
        wreg[t][1] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(wres, voff1, so, 2));
    };
    // in tile order, and kept so: the loop's wait counts are the worse of this order and its own
#pragma unroll
    for (int t = 0; t < T; ++t) {
        issue_w(t, t);
        __builtin_amdgcn_sched_barrier(0);
    }
    // the compiler does not track LDS-DMA: wait until only the 2T weight loads are outstanding
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * T));

    // ---- activations -> MFMA B operands (see gemv_stream_kernel) and the -sum(x) seed ----------
    uint32_t breg[2][4][8];
    f32x4 nsx = f32x4{0.f, 0.f, 0.f, 0.f};
    {
        int mr = 1;
        while (mr < rows) mr *= 2;
        const int xrow = mi & (mr - 1);
        const uint32_t xr_off = uint32_t(xrow) * 1024u + uint32_t(mg) * 128u;
        const uint32_t sw = uint32_t(xrow & 7);
        const bool live = mi < rows;
        const uint32_t sel_lo = live ? 0x05040100u : 0x0c0c0c0cu;
        const uint32_t sel_hi = live ? 0x07060302u : 0x0c0c0c0cu;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int wd = 0; wd < 4; ++wd) {
                const u32x4 lo = *reinterpret_cast<const u32x4*>(my_lds + xr_off + h * 512 + ((uint32_t(2 * wd) ^ sw) << 4));
                const u32x4 hi = *reinterpret_cast<const u32x4*>(my_lds + xr_off + h * 512 + ((uint32_t(2 * wd + 1) ^ sw) << 4));
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    breg[h][wd][2 * r] = __builtin_amdgcn_perm(hi[r], lo[r], sel_lo);
                    breg[h][wd][2 * r + 1] = __builtin_amdgcn_perm(hi[r], lo[r], sel_hi);
                }
            }
        const uint32_t c = 0x80108010u;                   // fp16 pair of -2^-20
        const u32x4 a = u32x4{c, c, c, c};
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const u32x4 bb = u32x4{breg[h][0][e], breg[h][1][e], breg[h][2][e], breg[h][3][e]};
                nsx = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(a), as_f16x8(bb), nsx, 0, 0, 0);
            }
    }

    const uint32_t ww_off = uint32_t(lr) * 128u + (uint32_t(lc ^ lr) << 4);
    const uint32_t wr_off0 = uint32_t(mi) * 128u + (uint32_t((mg) ^ (mi & 7)) << 4);
    const uint32_t wr_off1 = uint32_t(mi) * 128u + (uint32_t((4 + mg) ^ (mi & 7)) << 4);
    const float gamma = R.gamma * 65536.f;               // times the 2^16 left in the partial sums
    typedef __attribute__((address_space(1))) __half* gh_ptr;
    // the output quad this thread owns in an item's epilogue: tile t = threadIdx.x / 64 of the item
    const int ot = int(threadIdx.x) >> 6;
    const uint32_t ycol = uint32_t(R.tile0) * 16u + 4u * uint32_t(mg);       // + 16 (first + ot)
    gh_ptr const yrow = (gh_ptr)(R.y + size_t(mi) * size_t(N));

    // One item of NT tiles starting at tile `first` of the run.  REFILL: each tile's registers are
    // loaded again at once with the tile T further on.
    auto item = [&](auto nt_tag, auto refill_tag, int first, int parity) {
        constexpr int NT = decltype(nt_tag)::value;
        constexpr bool REFILL = decltype(refill_tag)::value;
        f32x4 part[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            unsigned char* const reg_t = my_lds + (t & 1) * 2048;
            // Writing a tile to LDS and asking for the tile that takes its registers is a handful
            // of LDS, scalar and memory instructions; they run at raised priority so that they do
            // not queue behind the other wave's decode (measured: decode sweep 17.55 -> 17.2 us).
            if constexpr (REFILL) __builtin_amdgcn_s_setprio(3);
            *reinterpret_cast<u32x4*>(reg_t + ww_off) = wreg[t][0];
            *reinterpret_cast<u32x4*>(reg_t + 1024 + ww_off) = wreg[t][1];
            if constexpr (REFILL) {
                issue_w(first + T + t, t);
                __builtin_amdgcn_s_setprio(0);
                // the requests leave here, as soon as the registers are free: left to itself the
                // scheduler sinks all of an item's loads to its end, which costs two tiles of lead
                __builtin_amdgcn_sched_barrier(0);
            }
            f32x4 acc[3];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const u32x4 wv = *reinterpret_cast<const u32x4*>(reg_t + (h ? wr_off1 : wr_off0));
                // element e of each half-word sits at bits 2e, 2e+1; the mantissa bits 4..9 (classes
                // 0..2 -> accumulators) hold e = 2,3,4 as loaded, e = 0,1 after << 4 and e = 5,6,7 after >> 6
                const u32x4 sh[3] = {wv << 4, wv, wv >> 6};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int src = e < 2 ? 0 : (e < 5 ? 1 : 2);
                    const int j = e < 2 ? e : (e < 5 ? e - 2 : e - 5);
                    const uint32_t mask = 0x00300030u << (2 * j);
                    const u32x4 a = sh[src] & mask;
                    const u32x4 bb = u32x4{breg[h][0][e], breg[h][1][e], breg[h][2][e], breg[h][3][e]};
                    // first product of an accumulator: class 0 starts from the -sum(x) seed, the others from zero
                    const f32x4 c0 = (h == 0 && (e == 0 || e == 1 || e == 4)) ? (j == 0 ? nsx : f32x4{0.f, 0.f, 0.f, 0.f}) : acc[j];
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(a), as_f16x8(bb), c0, 0, 0, 0);
                }
            }
            // the three classes carry 2^-20, 2^-18 and 2^-16: two fused multiply-adds leave the sum at
            // 2^-16, and that power of two goes into the scale of the epilogue (exact, same roundings)
            part[t] = __builtin_elementwise_fma(__builtin_elementwise_fma(acc[0], f32x4{4.f, 4.f, 4.f, 4.f}, acc[1]),
                                                f32x4{4.f, 4.f, 4.f, 4.f}, acc[2]);
        }
        // split-K: partial sums into this wave's set `parity`, one LDS-only barrier, fixed-order sum
        unsigned char* const red = my_lds + 4096 + parity * (T * 1024);
#pragma unroll
        for (int t = 0; t < NT; ++t) reinterpret_cast<f32x4*>(red + t * 1024)[lane] = part[t];
        __builtin_amdgcn_s_waitcnt(0xF | (0x3 << 14) | (0x7 << 4));
        __builtin_amdgcn_s_barrier();
        if (ot < NT) {
            f32x4 v[8];
#pragma unroll
            for (int w = 0; w < 8; ++w)
                v[w] = (w < NW) ? reinterpret_cast<const f32x4*>(lds_raw + w * kStride + 4096 + parity * (T * 1024) + ot * 1024)[lane]
                                : f32x4{0.f, 0.f, 0.f, 0.f};
            const f32x4 s = ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
            if (mi < rows) {
                const f16x2 lo = {(_Float16)(gamma * s[0]), (_Float16)(gamma * s[1])};
                const f16x2 hi = {(_Float16)(gamma * s[2]), (_Float16)(gamma * s[3])};
                *(__attribute__((address_space(1))) u32x2*)(yrow + (ycol + 16u * uint32_t(first + ot))) =
                    u32x2{__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
            }
        }
    };

    const int n_items = (ntiles + T - 1) / T;
    int i = 0;
    for (; i + 1 < n_items; ++i)
        item(std::integral_constant<int, T>{}, std::true_type{}, i * T, i & 1);
    const int rem = ntiles - i * T;                        // 1 .. T tiles are left
    if (T == 1 || rem == 1) item(std::integral_constant<int, 1>{}, std::false_type{}, i * T, i & 1);
    else if (T == 2 || rem == 2) item(std::integral_constant<int, (T >= 2 ? 2 : 1)>{}, std::false_type{}, i * T, i & 1);
    else item(std::integral_constant<int, T>{}, std::false_type{}, i * T, i & 1);
}

// ------------------------------------------------------------------------------------------
// Long-K form of the lean kernel: 4096 < K <= 16384 and at most T tiles per workgroup, i.e. the
// lone down projection of a block at decode batch sizes (11008 -> 4096, 14336 -> 4096), where a
// workgroup's whole share is one or two tiles and the time is a chain of memory round trips unless
// they overlap.  Wave w owns the K slices w, w + 8, w + 16, w + 24 ("passes").  All of a pass's
// data -- the activation slice by LDS-DMA, the T tile slices of weights into one of two register
// sets -- is requested while the pass before it is decoded, so the chain is one round trip plus
// the decodes:
//     x(0), W(0), W(1) | build(0) | x(1) | decode(0) | wait all | build(1) | W(2), x(2) | decode(1) | ...
// The accumulators of the T tiles stay in registers over all passes (three position classes each),
// the -sum(x) seeds of the passes add up in one accumulator, and the waves exchange partial sums
// once, at the end.  The LDS-DMA requests are inline assembly: for a transfer it knows of, the
// compiler drains the memory pipeline before every later LDS access, which would undo the overlap;
// every wait for them is an explicit s_waitcnt (and since the compiler's own count of outstanding
// loads starts afresh at each of those, the weight loads issued after it are waited for exactly).
constexpr int kLongMaxPasses = 4;
constexpr int kLongWaveLds = kWaveLds + 2048;     // 16 KB of activation staging + one tile slice

template <int T>
__global__ void __launch_bounds__(512)
gemv_longk_kernel(LeanBatch b)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int NW = blockDim.x >> 6;
    unsigned char* const my_lds = lds_raw + wave * kLongWaveLds;
    unsigned char* const tile_buf = my_lds + kWaveLds;
    typedef const __attribute__((address_space(1))) unsigned char* gbytes;

    const WgRec& R = b.rec[blockIdx.x];
    const int K = R.K, N = R.N, rows = R.Mrem, ntiles = R.ntiles;
    const int slices = (K + kSliceK - 1) / kSliceK;
    const int P = __builtin_amdgcn_readfirstlane((slices - wave + NW - 1) / NW);   // passes of this wave, >= 1
    const uint32_t row_bytes = uint32_t(K) >> 2;
    const uint32_t tile_bytes = 16u * row_bytes;

    const int lr = lane >> 3, lc = lane & 7;   // load mapping: row of the half tile, chunk of the slice
    const int mi = lane & 15, mg = lane >> 4;  // MFMA mapping: row / activation column, k group

    // ---- activations of slice wave + NW * p -> staging, swizzled (lane l fetches piece l ^ (r & 7) of row r)
    const uint32_t stage_addr = uint32_t(uintptr_t((const __attribute__((address_space(3))) unsigned char*)my_lds));
    auto dma16 = [&](gbytes src, uint32_t lds_base) {       // lane l: 16 bytes from src (per lane) to lds_base + 16 l
        const uint32_t base = __builtin_amdgcn_readfirstlane(lds_base);
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(base) : "memory");
    };
    auto stage_x = [&](int p) {
        const int sl = wave + NW * p;
        const size_t row_stride = size_t(K) * 2;
        gbytes src = (gbytes)(R.x + size_t(sl) * (kSliceK * 2));
        if ((sl + 1) * kSliceK <= K) {                      // the whole slice lies inside K
            const uint32_t lane16 = uint32_t(lane) << 4;
#pragma unroll 1
            for (int r = 0; r < rows; ++r) {
                dma16(src + (lane16 ^ (uint32_t(r & 7) << 4)), stage_addr + uint32_t(r) * 1024u);
                src += row_stride;
            }
        } else {
#pragma unroll 1
            for (int r = 0; r < rows; ++r) {
                const int kk = (lane ^ (r & 7)) << 3;      // first of this lane's 8 activations within the slice
                if (sl * kSliceK + kk < K) {
                    dma16(src + uint32_t(kk) * 2u, stage_addr + uint32_t(r) * 1024u);
                } else {
                    *reinterpret_cast<u32x4*>(my_lds + r * 1024 + (uint32_t(lane) << 4)) = u32x4{0u, 0u, 0u, 0u};
                }
                src += row_stride;
            }
        }
    };

    // ---- weights: the T tile slices of a pass into register set `set`
    const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(R.W), 0, uint32_t(ntiles) * tile_bytes, 0x00020000);
    u32x4 wreg[2][T][2];
    auto issue_w = [&](auto set_tag, int p) {
        constexpr int SET = decltype(set_tag)::value;
        uint32_t chunk = uint32_t(wave + NW * p) * 8u + uint32_t(lc);
        if (chunk >= (uint32_t(K) >> 6)) chunk = 0;        // past K: multiplied by zero activations
        const uint32_t voff0 = uint32_t(lr) * row_bytes + chunk * 16u;
        const uint32_t voff1 = voff0 + 8u * row_bytes;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const uint32_t so = uint32_t(t < ntiles ? t : ntiles - 1) * tile_bytes;   // past the run: its last tile again
            wreg[SET][t][0] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(wres, voff0, so, 2));   // 2: nt
            wreg[SET][t][1] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(wres, voff1, so, 2));
        }
    };

    // ---- staged activations -> MFMA B operands (as in gemv_lean_kernel); the pass's -sum(x) goes into nsx
    uint32_t breg[2][4][8];
    f32x4 nsx = f32x4{0.f, 0.f, 0.f, 0.f};
    int mr = 1;
    while (mr < rows) mr *= 2;
    const int xrow = mi & (mr - 1);
    const uint32_t xr_off = uint32_t(xrow) * 1024u + uint32_t(mg) * 128u;
    const uint32_t sw = uint32_t(xrow & 7);
    const bool live = mi < rows;
    const uint32_t sel_lo = live ? 0x05040100u : 0x0c0c0c0cu;
    const uint32_t sel_hi = live ? 0x07060302u : 0x0c0c0c0cu;
    auto build = [&]() {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int wd = 0; wd < 4; ++wd) {
                const u32x4 lo = *reinterpret_cast<const u32x4*>(my_lds + xr_off + h * 512 + ((uint32_t(2 * wd) ^ sw) << 4));
                const u32x4 hi = *reinterpret_cast<const u32x4*>(my_lds + xr_off + h * 512 + ((uint32_t(2 * wd + 1) ^ sw) << 4));
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    breg[h][wd][2 * r] = __builtin_amdgcn_perm(hi[r], lo[r], sel_lo);
                    breg[h][wd][2 * r + 1] = __builtin_amdgcn_perm(hi[r], lo[r], sel_hi);
                }
            }
        const uint32_t c = 0x80108010u;                   // fp16 pair of -2^-20
        const u32x4 a = u32x4{c, c, c, c};
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const u32x4 bb = u32x4{breg[h][0][e], breg[h][1][e], breg[h][2][e], breg[h][3][e]};
                nsx = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(a), as_f16x8(bb), nsx, 0, 0, 0);
            }
        // the staging area may be written again: every read above has returned
        __builtin_amdgcn_s_waitcnt(0xF | (0x3 << 14) | (0x7 << 4));      // lgkmcnt(0)
    };

    // ---- one pass of the T tiles from register set `set` into the tiles' accumulators
    const uint32_t ww_off = uint32_t(lr) * 128u + (uint32_t(lc ^ lr) << 4);
    const uint32_t wr_off0 = uint32_t(mi) * 128u + (uint32_t((mg) ^ (mi & 7)) << 4);
    const uint32_t wr_off1 = uint32_t(mi) * 128u + (uint32_t((4 + mg) ^ (mi & 7)) << 4);
    f32x4 acc[T][3];
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
        for (int j = 0; j < 3; ++j) acc[t][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    auto decode = [&](auto set_tag) {
        constexpr int SET = decltype(set_tag)::value;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            *reinterpret_cast<u32x4*>(tile_buf + ww_off) = wreg[SET][t][0];
            *reinterpret_cast<u32x4*>(tile_buf + 1024 + ww_off) = wreg[SET][t][1];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const u32x4 wv = *reinterpret_cast<const u32x4*>(tile_buf + (h ? wr_off1 : wr_off0));
                // element e of each half-word sits at bits 2e, 2e+1; the mantissa bits 4..9 (classes
                // 0..2 -> accumulators) hold e = 2,3,4 as loaded, e = 0,1 after << 4 and e = 5,6,7 after >> 6
                const u32x4 sh[3] = {wv << 4, wv, wv >> 6};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int src = e < 2 ? 0 : (e < 5 ? 1 : 2);
                    const int j = e < 2 ? e : (e < 5 ? e - 2 : e - 5);
                    const uint32_t mask = 0x00300030u << (2 * j);
                    const u32x4 a = sh[src] & mask;
                    const u32x4 bb = u32x4{breg[h][0][e], breg[h][1][e], breg[h][2][e], breg[h][3][e]};
                    acc[t][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(a), as_f16x8(bb), acc[t][j], 0, 0, 0);
                }
            }
        }
    };
    using Set0 = std::integral_constant<int, 0>;
    using Set1 = std::integral_constant<int, 1>;

    // ---- prologue: x(0), W(0), W(1) requested at once
    stage_x(0);
    issue_w(Set0{}, 0);
    if (P > 1) {
        issue_w(Set1{}, 1);
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(4 * T));      // x(0) is in
        build();
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * T));      // W(0) is in
        stage_x(1);
    } else {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * T));
        build();
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    }
    for (int p = 0; p < P; p += 2) {
        decode(Set0{});                                    // pass p
        if (p + 1 < P) {
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));      // x(p + 1) and W(p + 1) are in
            build();
            if (p + 2 < P) {
                issue_w(Set0{}, p + 2);
                stage_x(p + 2);
            }
            decode(Set1{});                                // pass p + 1
            if (p + 2 < P) {
                __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
                build();
                if (p + 3 < P) {
                    issue_w(Set1{}, p + 3);
                    stage_x(p + 3);
                }
            }
        }
    }

    // ---- split-K: partial sums (at 2^-16, see gemv_lean_kernel) into the staging area, one barrier, fixed-order sum
    const float gamma = R.gamma * 65536.f;
    typedef __attribute__((address_space(1))) __half* gh_ptr;
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const f32x4 four = f32x4{4.f, 4.f, 4.f, 4.f};
        const f32x4 part = __builtin_elementwise_fma(__builtin_elementwise_fma(acc[t][0] + nsx, four, acc[t][1]), four, acc[t][2]);
        reinterpret_cast<f32x4*>(my_lds + t * 1024)[lane] = part;
    }
    __builtin_amdgcn_s_waitcnt(0xF | (0x3 << 14) | (0x7 << 4));
    __builtin_amdgcn_s_barrier();
    const int ot = int(threadIdx.x) >> 6;
    if (ot < T && ot < ntiles) {
        f32x4 v[8];
#pragma unroll
        for (int w = 0; w < 8; ++w)
            v[w] = (w < NW) ? reinterpret_cast<const f32x4*>(lds_raw + w * kLongWaveLds + ot * 1024)[lane]
                            : f32x4{0.f, 0.f, 0.f, 0.f};
        const f32x4 s = ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
        if (mi < rows) {
            gh_ptr const yrow = (gh_ptr)(R.y + size_t(mi) * size_t(N));
            const uint32_t ycol = uint32_t(R.tile0 + ot) * 16u + 4u * uint32_t(mg);
            const f16x2 lo = {(_Float16)(gamma * s[0]), (_Float16)(gamma * s[1])};
            const f16x2 hi = {(_Float16)(gamma * s[2]), (_Float16)(gamma * s[3])};
            *(__attribute__((address_space(1))) u32x2*)(yrow + ycol) =
                u32x2{__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
        }
    }
}

using KernelFn = void (*)(GemvBatch);

template <bool MULTI>
KernelFn pick_kernel_t(int T)
{
    switch (T) {
        case 1: return gemv_kernel<1, MULTI>;
        case 2: return gemv_kernel<2, MULTI>;
        case 3: return gemv_kernel<3, MULTI>;
        default: return gemv_kernel<4, MULTI>;
    }
}

KernelFn pick_kernel(int T, bool multi)
{
    return multi ? pick_kernel_t<true>(T) : pick_kernel_t<false>(T);
}

template <bool MULTI, bool PASSES>
KernelFn pick_stream_t(int T)
{
    switch (T) {
        case 1: return gemv_stream_kernel<1, MULTI, PASSES, 1>;
        case 2: return gemv_stream_kernel<2, MULTI, PASSES, 1>;
        case 3: return gemv_stream_kernel<3, MULTI, PASSES, 1>;
        default: return gemv_stream_kernel<4, MULTI, PASSES, 1>;
    }
}

// units: scale units per 512-weight slice, 2 (256 weights each) or 4 (128 each, at most 2 tiles per item)
KernelFn pick_stream_gs(int T, bool passes, int units)
{
    if (units == 4) {
        if (T == 1) return passes ? gemv_stream_kernel<1, true, true, 1, 4> : gemv_stream_kernel<1, true, false, 1, 4>;
        return passes ? gemv_stream_kernel<2, true, true, 1, 4> : gemv_stream_kernel<2, true, false, 1, 4>;
    }
    switch (T) {
        case 1: return passes ? gemv_stream_kernel<1, true, true, 1, 2> : gemv_stream_kernel<1, true, false, 1, 2>;
        case 2: return passes ? gemv_stream_kernel<2, true, true, 1, 2> : gemv_stream_kernel<2, true, false, 1, 2>;
        default: return passes ? gemv_stream_kernel<3, true, true, 1, 2> : gemv_stream_kernel<3, true, false, 1, 2>;
    }
}

KernelFn pick_stream(int T, bool multi, bool passes, int nb)
{
    if (nb == 2) {                                         // two row blocks: T <= 2
        if (passes) return T == 1 ? gemv_stream_kernel<1, true, true, 2> : gemv_stream_kernel<2, true, true, 2>;
        if (T == 1) return multi ? gemv_stream_kernel<1, true, false, 2> : gemv_stream_kernel<1, false, false, 2>;
        return multi ? gemv_stream_kernel<2, true, false, 2> : gemv_stream_kernel<2, false, false, 2>;
    }
    if (passes) return multi ? pick_stream_t<true, true>(T) : pick_stream_t<false, true>(T);
    return multi ? pick_stream_t<true, false>(T) : pick_stream_t<false, false>(T);
}

int pow2_at_least(int v)
{
    int r = 1;
    while (r < v) r *= 2;
    return r;
}

constexpr int kMaxLds = 8 * kWaveLds;    // most dynamic LDS any launch asks for (8 waves, one item)

// Launch policy.  One 16-row job alone: 8-wave groups, one per CU, one item each while that
// covers the matrix.  Several jobs: 4-wave groups (two passes over K = 4096), two per CU, so
// that one group's wait for HBM overlaps the other's arithmetic, each looping over its items.
struct GemvPolicy {
    int nw_single = 8, nw_grouped = 4;
    int grid_cap = 512;                 // resident workgroups of the grouped form (2 per CU)
    int t_grouped = 0;                  // 0: pick from the tile count
    int stream = 3;                     // bit 0: stream form for one job, bit 1: for several
    int stream_groups = 256;            // workgroups of the stream form (one per CU)
    int two_blocks = 1;                 // jobs of more than 16 rows go in blocks of 32 (two row blocks per wave)
    double start_up_per_row = 0.15;     // stream form: start-up of a pass in tiles per activation row
    double pass_start = 1.5;            // stream form: wait of every pass but the first for its activations, in tiles
    int item_cost = 1;                  // stream form: allocation counts items, not only tiles
    double item_first = 2.1;            // cost of the first tile of an item, in average tiles
    double tile_extra = 0.43;           // cost of each further tile of an item
    int t_stream = 0;                   // stream form: cap on tiles per item (0: none)
    int long_k_min_run = 3;             // K > 4096 streams if the call averages this many tile passes per workgroup
    int lean = 1;                       // launches the lean kernel can take go to it
    int longk = 1;                      // lone calls with 4096 < K <= 16384 and at most two tiles per workgroup: long-K form
};
const GemvPolicy g_policy{};   // fixed in the library; development builds patch this line to try other values

constexpr int kStreamWaves = 8;         // waves of a stream-form workgroup when K >= 4096
constexpr int kStreamMaxPasses = 8;     // passes over K the stream form takes: K <= 32768
constexpr int kStreamMaxRun = 32;       // tiles of a run whose sums fit the 32 KB of LDS left over

using LeanFn = void (*)(LeanBatch);

LeanFn pick_lean(int T)
{
    switch (T) {
        case 1: return gemv_lean_kernel<1>;
        case 2: return gemv_lean_kernel<2>;
        default: return gemv_lean_kernel<3>;
    }
}

// Launch of the lean kernel: wg[j] workgroups for job j, each with a run of consecutive tiles
// (the first tiles % wg[j] of them one tile longer), written out as one record per workgroup.
hipError_t launch_lean(const GemvBatch& b, const int* wg, int NW, int T, hipStream_t s)
{
    LeanBatch lb;
    int grid = 0;
    for (int j = 0; j < b.count; ++j) {
        const GemvJob& J = b.job[j];
        const int per = J.tiles / wg[j], plus = J.tiles % wg[j];
        const size_t tile_bytes = size_t(16) * (size_t(J.K) / 4);
        for (int g = 0; g < wg[j]; ++g) {
            WgRec& r = lb.rec[grid++];
            r.tile0 = g * per + (g < plus ? g : plus);
            r.ntiles = per + (g < plus ? 1 : 0);
            r.W = reinterpret_cast<const unsigned char*>(J.W) + size_t(r.tile0) * tile_bytes;
            r.x = reinterpret_cast<const unsigned char*>(J.x);
            r.y = J.y;
            r.gamma = J.gamma;
            r.K = J.K; r.N = J.N; r.Mrem = J.Mrem;
            r.pad[0] = r.pad[1] = r.pad[2] = r.pad[3] = 0;
        }
    }
    LeanFn fn = pick_lean(T);
    static bool lds_raised[kMaxDevices][4];
    const int dev = device_slot();
    if (dev < 0 || !lds_raised[dev][T]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 8 * stream_wave_lds(3));
        if (e != hipSuccess) return e;
        if (dev >= 0) lds_raised[dev][T] = true;
    }
    hipLaunchKernelGGL(fn, dim3(grid), dim3(NW * 64), size_t(NW) * stream_wave_lds(T), s, lb);
    return hipGetLastError();
}

LeanFn pick_longk(int T)
{
    return T == 1 ? gemv_longk_kernel<1> : gemv_longk_kernel<2>;
}

// Calls in which every GEMM has 4096 < K <= 16384 and N a multiple of 16, and which hold at most two
// tiles per workgroup in all (the lone down projection of a block: 11008 -> 4096, 14336 -> 4096):
// the long-K form of the lean kernel, one record per workgroup with its one or two tiles.  Returns
// false, and launches nothing, for any other call.
bool launch_longk(const GemmDesc* jobs, int count, hipStream_t s, hipError_t* err)
{
    int64_t tiles_total = 0;
    for (int i = 0; i < count; ++i) {
        const GemmDesc& d = jobs[i];
        const int64_t slices = (d.K + kSliceK - 1) / kSliceK;
        if (slices <= kStreamWaves || slices > int64_t(kStreamWaves) * kLongMaxPasses || (d.N & 15) != 0) return false;
        tiles_total += ((d.M + 15) / 16) * (d.N / 16);
        if (tiles_total > 2 * kLeanMaxGroups) return false;
    }
    const int T = tiles_total <= kLeanMaxGroups ? 1 : 2;
    int64_t groups = 0;
    for (int i = 0; i < count; ++i) groups += ((jobs[i].M + 15) / 16) * ((jobs[i].N / 16 + T - 1) / T);
    if (groups > kLeanMaxGroups) return false;
    LeanBatch lb;
    int grid = 0;
    for (int i = 0; i < count; ++i) {
        const GemmDesc& d = jobs[i];
        const int tiles = int(d.N / 16);
        const size_t tile_bytes = size_t(16) * (size_t(d.K) / 4);
        for (int64_t m0 = 0; m0 < d.M; m0 += 16) {
            for (int t0 = 0; t0 < tiles; t0 += T) {
                WgRec& r = lb.rec[grid++];
                r.tile0 = t0;
                r.ntiles = tiles - t0 < T ? tiles - t0 : T;
                r.W = reinterpret_cast<const unsigned char*>(d.W) + size_t(t0) * tile_bytes;
                r.x = reinterpret_cast<const unsigned char*>(d.x + m0 * d.K);
                r.y = d.y + m0 * d.N;
                r.gamma = d.gamma;
                r.K = int(d.K); r.N = int(d.N);
                r.Mrem = int(d.M - m0 < 16 ? d.M - m0 : 16);
                r.pad[0] = r.pad[1] = r.pad[2] = r.pad[3] = 0;
            }
        }
    }
    LeanFn fn = pick_longk(T);
    static bool lds_raised[kMaxDevices][3];
    const int dev = device_slot();
    if (dev < 0 || !lds_raised[dev][T]) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, kStreamWaves * kLongWaveLds);
        if (e != hipSuccess) { *err = e; return true; }
        if (dev >= 0) lds_raised[dev][T] = true;
    }
    hipLaunchKernelGGL(fn, dim3(grid), dim3(kStreamWaves * 64), size_t(kStreamWaves) * kLongWaveLds, s, lb);
    *err = hipGetLastError();
    return true;
}

// Stream form: one job per workgroup, a run of consecutive tiles each.  Workgroups are dealt
// out to the jobs so that all finish together (see run_cost below); spare ones go to the job
// with the costliest runs, one by one.  Returns hipErrorInvalidValue without launching if a multi-pass job's
// runs would not fit the LDS (the caller then uses the general kernel).
hipError_t launch_stream(GemvBatch& b, int max_slices, int nb, hipStream_t s, int gs = 0)
{
    const GemvPolicy pol = g_policy;
    const int NW = max_slices < kStreamWaves ? max_slices : kStreamWaves;
    auto passes = [&](int j) { return (b.job[j].slices + NW - 1) / NW; };
    int64_t total_tiles = 0;
    bool multi_pass = false;
    for (int j = 0; j < b.count; ++j) {
        total_tiles += b.job[j].tiles;
        multi_pass |= passes(j) > 1;
    }
    // One workgroup of 8 waves per CU; with shorter K (fewer waves per workgroup) as many more
    // workgroups, so that a CU still runs 8 waves (K = 1024: 1024 workgroups of 2 waves).
    const int64_t g_max = int64_t(pol.stream_groups) * (kStreamWaves / NW);
    const int G = total_tiles < g_max ? int(total_tiles) : int(g_max);
    // Time of a workgroup in tile units: passes x (run time + start-up), see tl_deal.hpp.  The
    // start-up of a pass is fetching the activation slice (1 KB per row and wave through the same
    // address path as the weights) and building the operands: measured about 0.15 tiles per
    // activation row; a job of several passes pays part of that round trip in every pass but the
    // first (pass_start tiles).  A run is worked off in items of up to t_max tiles, and an item
    // costs its latency and barrier once: measured (block launch, runs of 15 ... 19 tiles) 1.0 us
    // for the first tile of an item and 0.2 us for each further one, i.e. 2.1 and 0.43 in units
    // of an average tile.
    const DealModel model{(nb == 2 || gs == 4) ? 2 : 3, pol.item_cost != 0, pol.item_first, pol.tile_extra};
    DealJob dj[kMaxJobs];
    for (int j = 0; j < b.count; ++j) {
        const int rows = b.job[j].Mrem < 16 * nb ? b.job[j].Mrem : 16 * nb;
        dj[j] = DealJob{b.job[j].tiles, passes(j),
                        pol.start_up_per_row * double(rows) + (passes(j) > 1 ? pol.pass_start : 0.0)};
    }
    int wg[kMaxJobs];
    deal_workgroups(model, dj, b.count, G, wg);
    int run = 1;                                           // longest run of tiles of a workgroup
    for (int j = 0; j < b.count; ++j) {
        const int r = (b.job[j].tiles + wg[j] - 1) / wg[j];
        if (passes(j) > 1 && r > kStreamMaxRun / nb) return hipErrorInvalidValue;   // 1 KB of kept sums per tile and row block
        if (r > run) run = r;
    }
    // Tiles per item.  Measured: items of 3 tiles stream 3-4 % faster than items of 4 (6 KB
    // against 8 KB requested per wave at a time; with more in flight the memory system slows
    // down), a run of 4 goes best as 2 + 2 (the second pair loads while the first is decoded),
    // and shorter runs are one item.
    int T = run <= 3 ? run : (run == 4 ? 2 : 3);
    if (T > NW) T = NW;                  // the epilogue gives every thread at most one output quad
    if (pol.t_stream > 0 && T > pol.t_stream) T = pol.t_stream;
    if (gs == 4 && T > 2) T = 2;         // scale units of 128 weights: 12 accumulators per tile (registers)
    if (nb == 2) {                       // two row blocks per job: at most 2 tiles per item (registers)
        if (T > 2) T = 2;
        if (2 * T > NW) T = NW / 2;
        if (T < 1) return hipErrorInvalidValue;
    }
    if (T < 1) T = 1;
    // The lean kernel takes the launch when every job has the same number of slices (one per wave),
    // N is a multiple of 16 throughout and the workgroups fit its record table.
    bool lean = pol.lean && !multi_pass && nb == 1 && gs == 0 && T <= 3;
    int total_groups = 0;
    for (int j = 0; j < b.count; ++j) {
        lean = lean && b.job[j].slices == NW && (b.job[j].N & 15) == 0;
        total_groups += wg[j];
    }
    if (lean && total_groups <= kLeanMaxGroups) return launch_lean(b, wg, NW, T, s);
    for (int j = 0; j < kMaxJobs; ++j) b.item0[j] = 0x7fffffff;
    int grid = 0;
    for (int j = 0; j < b.count; ++j) {
        b.item0[j] = grid;
        b.job[j].items = 0;
        b.job[j].run = b.job[j].tiles / wg[j];
        b.job[j].plus = b.job[j].tiles % wg[j];
        grid += wg[j];
    }
    const size_t lds = size_t(NW) * stream_wave_lds(T * nb) + (multi_pass ? size_t(kStreamMaxRun) * 1024 : 0);
    b.total_items = 0;                                 // the stream form has no item queue
    b.red_off = 0;
    b.pad = 0;
    const bool multi = gs != 0 || b.count > 1;         // the scaled form always reads the job table
    KernelFn fn = gs ? pick_stream_gs(T, multi_pass, gs) : pick_stream(T, multi, multi_pass, nb);
    static bool lds_raised[kMaxDevices][8][2][kTMax + 1];
    const int variant = gs == 4 ? (multi_pass ? 7 : 6)
                                : (gs ? (multi_pass ? 4 : 3) : (nb == 2 ? (multi_pass ? 5 : 2) : (multi_pass ? 1 : 0)));
    const int dev = device_slot();
    if (dev < 0 || !lds_raised[dev][variant][multi][T]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           8 * stream_wave_lds(T) + kStreamMaxRun * 1024);
        if (e != hipSuccess) return e;
        if (dev >= 0) lds_raised[dev][variant][multi][T] = true;
    }
    hipLaunchKernelGGL(fn, dim3(grid), dim3(NW * 64), lds, s, b);
    return hipGetLastError();
}

// Launch one batch (<= kMaxJobs jobs, tiles / slices / M filled in): sets items and grid.
hipError_t launch_batch(GemvBatch& b, bool grouped, bool stream_form, int nb, hipStream_t s)
{
    const GemvPolicy pol = g_policy;
    int64_t total_tiles = 0;
    int max_slices = 1;
    for (int j = 0; j < b.count; ++j) {
        total_tiles += b.job[j].tiles;
        if (b.job[j].slices > max_slices) max_slices = b.job[j].slices;
    }
    if (stream_form && max_slices <= kStreamWaves * kStreamMaxPasses && (pol.stream & (b.count > 1 ? 2 : 1))) {
        const hipError_t e = launch_stream(b, max_slices, nb, s);
        if (e != hipErrorInvalidValue) return e;           // else: runs too long for its LDS, general kernel
    }
    if (nb != 1) {
        // jobs of two row blocks exist for the stream form only: each goes on as two jobs of 16 rows
        GemvBatch h;
        h.count = 0;
        for (int j = 0; j < b.count; ++j) {
            for (int part = 0; part < 2; ++part) {
                const int rows = b.job[j].Mrem - 16 * part;
                if (rows <= 0) break;
                GemvJob q = b.job[j];
                q.x = b.job[j].x + size_t(16 * part) * size_t(q.K);
                q.y = b.job[j].y + size_t(16 * part) * size_t(q.N);
                q.Mrem = rows < 16 ? rows : 16;
                q.mr = pow2_at_least(q.Mrem);
                h.job[h.count++] = q;
                if (h.count == kMaxJobs) {
                    const hipError_t e = launch_batch(h, true, false, 1, s);
                    if (e != hipSuccess) return e;
                    h.count = 0;
                }
            }
        }
        return h.count ? launch_batch(h, true, false, 1, s) : hipSuccess;
    }
    int NW = grouped ? pol.nw_grouped : pol.nw_single;
    if (NW > max_slices) NW = max_slices;
    int resident = grouped ? pol.grid_cap : (NW <= 4 ? 512 : 256);
    int T = (grouped && pol.t_grouped) ? pol.t_grouped : int((total_tiles + resident - 1) / resident);
    if (T > kTMax) T = kTMax;
    if (T < 1) T = 1;
    int total_items = 0;
    for (int j = 0; j < kMaxJobs; ++j) b.item0[j] = 0x7fffffff;
    for (int j = 0; j < b.count; ++j) {
        b.job[j].items = (b.job[j].tiles + T - 1) / T;
        b.item0[j] = total_items;
        total_items += b.job[j].items;
    }
    b.total_items = total_items;
    // Workgroups that loop keep the reduction area behind the staging area; with 8 waves
    // that is more LDS than a CU has, so a looping launch uses 4-wave groups, two per CU.
    if (total_items > resident && NW > 4) { NW = 4; resident = 512; }
    const int grid = total_items < resident ? total_items : resident;
    const bool looping = total_items > grid;
    b.red_off = looping ? NW * kWaveLds : 0;
    const int lds = NW * kWaveLds + (looping ? T * NW * 1024 : 0);
    b.pad = 0;

    const bool multi = b.count > 1;
    KernelFn fn = pick_kernel(T, multi);
    // More than the default 64 KB of dynamic LDS needs the attribute; it is set once per
    // kernel instance and device (idempotent, so a race only repeats it).
    static bool lds_raised[kMaxDevices][2][kTMax + 1];
    const int dev = device_slot();
    if (dev < 0 || !lds_raised[dev][multi][T]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds);
        if (e != hipSuccess) return e;
        if (dev >= 0) lds_raised[dev][multi][T] = true;
    }
    hipLaunchKernelGGL(fn, dim3(grid), dim3(NW * 64), size_t(lds), s, b);
    return hipGetLastError();
}

}  // namespace

// Raises the dynamic-LDS limit of every kernel instance of this file on the current device (the
// launchers do it on first use otherwise).
hipError_t gemv_init()
{
    const int stream_lds = 8 * kWaveLds + kStreamMaxRun * 1024;
    auto raise = [](KernelFn fn, int bytes) {
        return hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    };
    for (int T = 1; T <= 2; ++T) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(pick_longk(T)), hipFuncAttributeMaxDynamicSharedMemorySize, kStreamWaves * kLongWaveLds);
        if (e != hipSuccess) return e;
    }
    for (int T = 1; T <= 3; ++T) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(pick_lean(T)), hipFuncAttributeMaxDynamicSharedMemorySize, 8 * stream_wave_lds(3));
        if (e != hipSuccess) return e;
    }
    for (int T = 1; T <= kTMax; ++T)
        for (int multi = 0; multi < 2; ++multi) {
            hipError_t e = raise(pick_kernel(T, multi != 0), kMaxLds);
            for (int passes = 0; passes < 2 && e == hipSuccess; ++passes) {
                e = raise(pick_stream(T, multi != 0, passes != 0, 1), stream_lds);
                if (e == hipSuccess && T <= 2) e = raise(pick_stream(T, multi != 0, passes != 0, 2), stream_lds);
                if (e == hipSuccess && T <= 3) e = raise(pick_stream_gs(T, passes != 0, 2), stream_lds);
                if (e == hipSuccess && T <= 2) e = raise(pick_stream_gs(T, passes != 0, 4), stream_lds);
            }
            if (e != hipSuccess) return e;
        }
    return hipSuccess;
}

bool gemv_supports(int64_t M, int64_t N, int64_t K)
{
    return M >= 1 && N >= 1 && K >= 64 && (K % 64) == 0 && K <= (int64_t(1) << 24) &&
           N <= (int64_t(1) << 24) && M <= (int64_t(1) << 20);
}

hipError_t launch_gemv_jobs(const GemmDesc* jobs, int count, hipStream_t s)
{
    if (g_policy.longk) {
        hipError_t e = hipSuccess;
        if (launch_longk(jobs, count, s, &e)) return e;
    }
    // A user job with M > 16 becomes ceil(M / 16) kernel jobs (blocks of 16 activation rows).
    int64_t blocks_total = 0;
    for (int i = 0; i < count; ++i) blocks_total += (jobs[i].M + 15) / 16;
    const bool grouped = blocks_total > 1;

    // Two batches fill side by side: jobs for the stream form and jobs for the general kernel.
    // K <= 4096 always streams.  Longer K streams in several passes, each of which starts with
    // a round trip to memory for the activations; that pays once the call holds enough work to
    // give every workgroup a run of a few tiles (e.g. the linears of a whole block), otherwise
    // the general kernel takes those jobs.
    int64_t call_tiles = 0;                                   // tiles of the whole call
    for (int i = 0; i < count; ++i) call_tiles += ((jobs[i].M + 15) / 16) * ((jobs[i].N + 15) / 16);
    // (measured: one job of 512 tiles is better off in the general kernel, 11008 -> 8192 at M = 1
    // 9.7 against 10.9 us; two jobs of 256 tiles stream better, 11008 -> 4096 at M = 32 16.1 against 20.3 us)
    const bool long_k_streams = call_tiles >= int64_t(g_policy.stream_groups) * g_policy.long_k_min_run ||
                                (blocks_total >= 2 && call_tiles >= int64_t(g_policy.stream_groups) * 2);
    // bs: stream form; bs2: stream form with jobs of up to 32 rows (two blocks of 16 per wave);
    // bg: general kernel
    GemvBatch bs, bs2, bg;
    bs.count = 0;
    bs2.count = 0;
    bg.count = 0;
    auto flush = [&](GemvBatch& b) -> hipError_t {
        if (b.count == 0) return hipSuccess;
        hipError_t e = launch_batch(b, grouped, &b != &bg, &b == &bs2 ? 2 : 1, s);
        b.count = 0;
        return e;
    };
    const bool stream_on = (g_policy.stream & 3) == 3;
    for (int i = 0; i < count; ++i) {
        const GemmDesc& d = jobs[i];
        const int slices = int((d.K + kSliceK - 1) / kSliceK);
        // more than 16 rows and one pass over K: blocks of 32 rows, decoded once for both halves
        const bool two_blocks = stream_on && g_policy.two_blocks && gemv_two_blocks(d.M, d.N, d.K);
        const int64_t mstep = two_blocks ? 32 : 16;
        for (int64_t m0 = 0; m0 < d.M; m0 += mstep) {
            GemvJob j;
            j.x = d.x + m0 * d.K;
            j.W = d.W;
            j.y = d.y + m0 * d.N;
            j.gamma = d.gamma;
            j.Mrem = int(d.M - m0 < mstep ? d.M - m0 : mstep);
            j.N = int(d.N); j.K = int(d.K);
            j.tiles = int((d.N + 15) / 16);
            j.items = 0;
            j.slices = slices;
            j.mr = pow2_at_least(j.Mrem < 16 ? j.Mrem : 16);
            j.run = j.plus = 0;
            j.scales = nullptr; j.hpg = 0; j.reserved = 0;
            const bool streams = j.slices <= kStreamWaves ||
                                 (long_k_streams && j.slices <= kStreamWaves * kStreamMaxPasses);
            GemvBatch& b = two_blocks ? bs2 : (streams ? bs : bg);
            if (two_blocks && j.slices > kStreamWaves) {
                // several passes: the kept sums allow runs of kStreamMaxRun / 2 tiles, so a launch holds
                // at most that many tiles per workgroup
                int64_t held = j.tiles;
                for (int q = 0; q < b.count; ++q) held += b.job[q].tiles;
                if (b.count > 0 && held > int64_t(g_policy.stream_groups) * (kStreamMaxRun / 2)) {
                    hipError_t e = flush(b);
                    if (e != hipSuccess) return e;
                }
            }
            b.job[b.count++] = j;
            if (b.count == kMaxJobs) {
                hipError_t e = flush(b);
                if (e != hipSuccess) return e;
            }
        }
    }
    hipError_t e = flush(bs);
    if (e != hipSuccess) return e;
    e = flush(bs2);
    if (e != hipSuccess) return e;
    return flush(bg);
}

bool gemv_gs_supports(int64_t M, int64_t N, int64_t K, int64_t group)
{
    const int64_t slices = (K + kSliceK - 1) / kSliceK;
    // (the kernel addresses the scales with 32-bit byte offsets)
    if (((K + group - 1) / group) * N * 2 >= (int64_t(1) << 31)) return false;
    return gemv_supports(M, N, K) && group >= 128 && group % 128 == 0 && N >= 4 && N % 4 == 0 &&
           slices <= kStreamWaves * kStreamMaxPasses &&
           (slices <= kStreamWaves || (N + 15) / 16 <= int64_t(256) * kStreamMaxRun);
}

hipError_t launch_gemv_gs_jobs(const GemmGsDesc* jobs, int count, hipStream_t s)
{
    for (int i = 0; i < count; ++i)
        if (!gemv_gs_supports(jobs[i].M, jobs[i].N, jobs[i].K, jobs[i].group)) return hipErrorInvalidValue;
    // Jobs whose groups are multiples of 256 weights and jobs with odd multiples of 128 run in
    // different instances of the kernel; each kind shares launches, kMaxJobs blocks of 16
    // activation rows per launch.  A launch whose runs would not fit the LDS of a multi-pass
    // workgroup (launch_stream says so without launching) goes out as one launch per job.
    for (int units = 2; units <= 4; units += 2) {
        GemvBatch b;
        b.count = 0;
        int max_slices = 1;
        auto flush = [&]() -> hipError_t {
            if (b.count == 0) return hipSuccess;
            hipError_t e = launch_stream(b, max_slices, 1, s, units);
            if (e == hipErrorInvalidValue && b.count > 1) {
                // one launch per row block; a block alone fits by gemv_gs_supports
                e = hipSuccess;
                for (int q = 0; q < b.count && e == hipSuccess; ++q) {
                    GemvBatch one;
                    one.count = 1;
                    one.job[0] = b.job[q];
                    e = launch_stream(one, one.job[0].slices, 1, s, units);
                }
            }
            b.count = 0;
            max_slices = 1;
            return e;
        };
        for (int i = 0; i < count; ++i) {
            const GemmGsDesc& d = jobs[i];
            if ((d.group % 256 == 0 ? 2 : 4) != units) continue;
            const int slices = int((d.K + kSliceK - 1) / kSliceK);
            const int hpg = int(d.group / (kSliceK / units));
            for (int64_t m0 = 0; m0 < d.M; m0 += 16) {
                GemvJob j;
                j.x = d.x + m0 * d.K;
                j.W = d.W;
                j.y = d.y + m0 * d.N;
                j.gamma = 1.f;
                j.Mrem = int(d.M - m0 < 16 ? d.M - m0 : 16);
                j.N = int(d.N); j.K = int(d.K);
                j.tiles = int((d.N + 15) / 16);
                j.items = 0;
                j.slices = slices;
                j.mr = pow2_at_least(j.Mrem);
                j.run = j.plus = 0;
                j.scales = d.scales; j.hpg = hpg; j.reserved = 0;
                b.job[b.count++] = j;
                if (slices > max_slices) max_slices = slices;
                if (b.count == kMaxJobs) {
                    const hipError_t e = flush();
                    if (e != hipSuccess) return e;
                }
            }
        }
        const hipError_t e = flush();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_gemv_gs(const __half* x, const uint32_t* Wp, const __half* scales, int64_t group,
                          __half* y, int64_t M, int64_t N, int64_t K, hipStream_t s)
{
    const GemmGsDesc d{x, Wp, scales, y, M, N, K, group};
    return launch_gemv_gs_jobs(&d, 1, s);
}

hipError_t launch_gemv(const __half* x, const uint32_t* Wp, float gamma, __half* y,
                       int64_t M, int64_t N, int64_t K, hipStream_t s)
{
    GemmDesc d{x, Wp, y, gamma, M, N, K};
    return launch_gemv_jobs(&d, 1, s);
}

}  // namespace tl
