/*
 * tl.h -- C ABI of the ternary-linear library for MI355X (gfx950).
 *
 * The library computes the inference form of the ternary linear layer of
 * Spectra-1.1 (arXiv 2506.23025):
 *
 *     Y = X * (gamma * What)^T          (paper App. B, "Inference", steps 1-3)
 *
 * with X fp16 [M][K], What in {-1,0,+1} [N][K] kept in one of the packed forms
 * of paper Sec. 3 and a single fp16 scale gamma per matrix (paper Sec. 2.1).
 * Accumulation is fp32 and the output is fp16 with round-to-nearest-even
 * (paper App. G, "Precision-Preserving Accumulation").
 *
 * Conventions shared by every entry point
 *   - All functions return a tl_status and never throw, abort or print.
 *   - "host" pointers are ordinary CPU memory; "device" pointers are HBM
 *     addresses valid on the current HIP device.  The caller owns every
 *     buffer; the library allocates nothing.  The only state it keeps between calls is
 *     a set of once-per-device flags that record that a kernel's launch attribute (its
 *     dynamic-LDS limit) has been set; tl_init sets them all.  Results never depend on it.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Device entry points only enqueue work on that stream and return; they
 *     never synchronise.  Errors reported by the launch come back as
 *     TL_ERR_HIP.
 *   - Matrices are dense row-major.  Packed weights are row-major too: row n
 *     occupies tl_row_stride_bytes(fmt, K) bytes starting at
 *     n * tl_row_stride_bytes(fmt, K).
 */
#ifndef TL_H_
#define TL_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum tl_status {
    TL_OK = 0,
    TL_ERR_NULL = 1,        /* a required pointer is NULL                         */
    TL_ERR_SHAPE = 2,       /* M, N or K < 1, or a size product overflows          */
    TL_ERR_VALUE = 3,       /* weight outside {-1,0,1}, or an invalid packed code  */
    TL_ERR_ALIGN = 4,       /* device pointer not 16-byte aligned                  */
    TL_ERR_UNSUPPORTED = 5, /* unknown format / path, or path cannot run the shape */
    TL_ERR_HIP = 6          /* the HIP runtime reported an error on launch         */
} tl_status;

typedef enum tl_format {
    TL_FMT_2BIT = 0,   /* paper Sec. 3.1 with k = 16 digits per 32-bit word      */
    TL_FMT_1P6BIT = 1, /* 5 trits per byte, plain base 3 (see tl_pack_1p6bit)    */
    TL_FMT_1P6BIT_FX = 2, /* 5 trits per byte, the fixed-point code as the paper prints it
                            (see tl_pack_1p6bit_fx); same row geometry as TL_FMT_1P6BIT */
    TL_FMT_INT_RANGE_ = 0x7fffffff /* not a format: makes every non-negative int a value the type
                            can hold, so that an unknown code is reported, not undefined */
} tl_format;

/* Kernel choice for tl_ternary_gemm_path.  AUTO is what tl_ternary_gemm uses. */
typedef enum tl_path {
    TL_PATH_AUTO = 0,
    TL_PATH_GENERIC = 1, /* plain VALU kernel, any M, N, K                        */
    TL_PATH_GEMV = 2,    /* weight-streaming small-M kernel: M <= 16 per pass     */
    TL_PATH_MFMA = 3,    /* LDS-tiled fp16 MFMA prefill kernel                    */
    TL_PATH_INT_RANGE_ = 0x7fffffff /* not a path (see TL_FMT_INT_RANGE_)         */
} tl_path;

/* Human-readable name of a status code (static storage, never NULL). */
const char* tl_status_str(tl_status s);

/*
 * Bytes from the start of one packed row to the next.
 *   TL_FMT_2BIT  : 4 * ceil(K / 16)                  (one uint32 per 16 weights)
 *   TL_FMT_1P6BIT: ceil(K / 5) rounded up to 16      (one byte per 5 weights;
 *                  the bytes after the last code byte are zero and never decoded)
 * Returns 0 for K < 1 or an unknown format.
 */
size_t tl_row_stride_bytes(tl_format fmt, int64_t K);

/* N * tl_row_stride_bytes(fmt, K); 0 on bad arguments. */
size_t tl_packed_bytes(tl_format fmt, int64_t N, int64_t K);

/*
 * Ternarisation of a trained weight matrix, paper App. B "Forward Pass":
 *   gamma = eps + mean |W_ij|,   What_ij = round(min(max(W_ij / gamma, -1), 1)).
 * The mean and the quotient are taken in fp64; round is round-half-to-even (the paper does
 * not say which; ties have measure zero for trained weights).  Per tensor only.
 *   W     host, float [N][K] row-major, finite
 *   What  host, int8 [N][K], written with values in {-1,0,1} (ready for tl_pack_*)
 *   gamma            if not NULL: the scale as computed (fp64)
 *   gamma_fp16_bits  if not NULL: the same rounded to fp16 (round to nearest even), the
 *                    form tl_ternary_gemm takes
 * TL_ERR_VALUE if W holds a NaN or an infinity, or eps is negative or not finite.
 */
tl_status tl_quantize(const float* W, int64_t N, int64_t K, double eps, int8_t* What,
                      double* gamma, uint16_t* gamma_fp16_bits);

/*
 * 2-bit packing P of paper Sec. 3.1 with k = 16: digit d' = w + 1 in {0,1,2};
 * word i of a row holds weights 16i .. 16i+15, weight 16i+j in bits [2j+1:2j].
 * A short last word is filled with weight 0 (digit 1), as the paper prescribes.
 *   W   host, int8 [N][K] row-major, every value in {-1,0,1}
 *   out host, uint32 [N][ceil(K/16)], written completely
 * TL_ERR_VALUE if any weight is outside {-1,0,1} (out is then unspecified).
 */
tl_status tl_pack_2bit(const int8_t* W, int64_t N, int64_t K, uint32_t* out);

/*
 * 1.6-bit packing: the base-3 block code of paper Sec. 3.2 (k = 5 digits in one
 * byte) in its plain, unscaled little-endian form: byte b of a row holds weights
 * 5b .. 5b+4 as sum_i (w[5b+i] + 1) * 3^i, a value in [0, 242].  Missing weights
 * of the last byte count as 0 (digit 1).  Rows are tl_row_stride_bytes apart and
 * the stride padding is written as zero.
 *   W   host, int8 [N][K];  out host, uint8 [N][stride]
 */
tl_status tl_pack_1p6bit(const int8_t* W, int64_t N, int64_t K, uint8_t* out);

/*
 * The fixed-point 1.6-bit code exactly as printed in paper Sec. 3.2 / App. E
 * (k = 5, p = 8): digits big-endian, Nval = sum_j d'_j 3^(4-j), byte =
 * floor((Nval * 256 + 242) / 243).  Same row geometry as tl_pack_1p6bit.
 * Decoded by tl_unpack_1p6bit_fx with the multiply-by-3 digit extraction of
 * paper App. F, Alg. 1 (on the GPU: tl_unpack_dev / tl_ternary_gemm_1p6_fx with
 * TL_FMT_1P6BIT_FX).
 */
tl_status tl_pack_1p6bit_fx(const int8_t* W, int64_t N, int64_t K, uint8_t* out);
tl_status tl_unpack_1p6bit_fx(const uint8_t* packed, int64_t N, int64_t K, int8_t* W_out);

/*
 * Unpacking U (paper Sec. 3.1 "Unpacking/Decoding"; Sec. 3.2 for base 3) on the
 * host.  packed: host, layout as written by the packers.  W_out: host int8
 * [N][K].  TL_ERR_VALUE on a 2-bit code 3 or a 1.6-bit byte > 242.
 */
tl_status tl_unpack(tl_format fmt, const void* packed, int64_t N, int64_t K, int8_t* W_out);

/*
 * The same decode on the GPU: packed and W_out are device pointers.  Invalid
 * codes are not reported; a 2-bit code 3 decodes to +2 and a byte > 242 to the
 * digits of its value modulo 243.  Exists so that the device decode can be
 * compared byte for byte with the host one.
 */
tl_status tl_unpack_dev(tl_format fmt, const void* packed, int64_t N, int64_t K,
                        int8_t* W_out, void* stream);

/*
 * y[m][n] = fp16_rne( float(gamma) * sum_k x[m][k] * w[n][k] ),  fp32 accumulation.
 *   x       device, fp16 [M][K] row-major, 16-byte aligned
 *   Wpacked device, TL_FMT_2BIT layout, 16-byte aligned
 *   gamma_fp16_bits  the per-matrix scale as raw IEEE binary16 bits
 *   y       device, fp16 [M][N] row-major, 16-byte aligned; fully overwritten
 * Activations are expected to be finite.  A NaN in row m of x makes row m of y NaN (no other
 * row); an infinity in row m makes that row NaN where the exact result would be +-infinity,
 * because the fast kernels compute sum (w + 1) x - sum x (Sec. 3.1 stores w + 1).
 * Any M, N, K >= 1 is accepted; the library picks the kernel from the shape
 * (small M: weight-streaming kernel; large M: LDS-tiled MFMA kernel; shapes the
 * fast kernels cannot take: the generic kernel).  Results are deterministic:
 * no atomics, fixed reduction order.  Behaviour on a 2-bit code 3 is memory-safe
 * but otherwise unspecified.
 */
tl_status tl_ternary_gemm(const void* x, const void* Wpacked, uint16_t gamma_fp16_bits,
                          void* y, int64_t M, int64_t N, int64_t K, void* stream);

/*
 * Optional.  Prepares every kernel of the library on the current HIP device (their limits for
 * dynamically sized LDS) so that no later call has to: without it each kernel instance does
 * this the first time it is launched.  Call it once per device, e.g. before capturing the
 * library's calls into a HIP graph.  Idempotent; allocates nothing; TL_ERR_HIP if the runtime
 * refuses.
 */
tl_status tl_init(void);

/*
 * The kernel tl_ternary_gemm (TL_PATH_AUTO) runs for a shape: TL_PATH_GEMV, TL_PATH_MFMA or
 * TL_PATH_GENERIC; TL_PATH_AUTO (0) if M, N or K is not a valid size.  A pure function of the
 * three numbers (host side, touches no GPU): the library's cost models of its two fast
 * kernels decide between them where both can run the shape.
 */
tl_path tl_ternary_gemm_which(int64_t M, int64_t N, int64_t K);

/* Same, with the kernel forced.  TL_ERR_UNSUPPORTED if `path` cannot run the shape. */
tl_status tl_ternary_gemm_path(const void* x, const void* Wpacked, uint16_t gamma_fp16_bits,
                               void* y, int64_t M, int64_t N, int64_t K, void* stream,
                               tl_path path);

/*
 * Several independent products in one call: the linears of a transformer block (the unit
 * the paper's kernel benchmark is quoted on, App. G "performance benchmark"), or any list
 * of (x, W, gamma, y).  Each job has the contract of tl_ternary_gemm.  No job reads what
 * another writes, and jobs must not alias
 * each other's outputs; they are enqueued in as few kernel launches as possible (jobs that
 * go to the small-M kernel share launches, 16 blocks of 16 activation rows per launch) and
 * may run concurrently.  `jobs` is host memory, read before the call returns.
 */
typedef struct tl_gemm_job {
    const void* x;            /* device, fp16 [M][K]                */
    const void* Wpacked;      /* device, TL_FMT_2BIT                */
    void* y;                  /* device, fp16 [M][N]                */
    int64_t M, N, K;
    uint16_t gamma_fp16_bits;
} tl_gemm_job;

tl_status tl_ternary_gemm_grouped(const tl_gemm_job* jobs, int64_t count, void* stream);

/* Same contract for weights in the TL_FMT_1P6BIT layout of tl_pack_1p6bit. */
tl_status tl_ternary_gemm_1p6(const void* x, const void* Wpacked, uint16_t gamma_fp16_bits,
                              void* y, int64_t M, int64_t N, int64_t K, void* stream);

/*
 * Same contract for weights in the TL_FMT_1P6BIT_FX layout of tl_pack_1p6bit_fx: the
 * 1.6-bit code of paper Sec. 3.2 as printed, decoded on the GPU by the multiply-by-3 digit
 * extraction of App. F, Alg. 1 (the paper leaves a GPU kernel for this format as future
 * work, Sec. 3.3 "Limitations").
 */
tl_status tl_ternary_gemm_1p6_fx(const void* x, const void* Wpacked, uint16_t gamma_fp16_bits,
                                 void* y, int64_t M, int64_t N, int64_t K, void* stream);

/*
 * The same product with one fp16 scale per group of `group` consecutive weights along K and
 * per output row, in place of the single gamma:
 *     y[m][n] = sum_g scales[g][n] * ( sum_{k in group g} x[m][k] * w[n][k] )
 * (paper Sec. 3.3, CPU inference: the 2-bit block format keeps one fp16 scale per block of
 * 256 weights; GPU kernel appendix: the dequantised fragments are scaled by quantisation
 * scales held in a separate buffer).  `scales` is a device pointer to fp16
 * [ceil(K / group)][N], 16-byte aligned; the last group may be short.  x, Wpacked (2-bit
 * format), y, stream, accumulation and rounding as for tl_ternary_gemm.  `group` must be a
 * multiple of 16 (TL_ERR_SHAPE otherwise).  group % 128 == 0, K % 64 == 0 and N % 4 == 0 run
 * in the weight-streaming small-M kernel (M in blocks of 16 rows; multiples of 256 a little
 * faster than odd multiples of 128); everything else in the generic kernel on the vector ALUs.
 * Nothing is allocated; the call is asynchronous on `stream`.
 */
tl_status tl_ternary_gemm_gs(const void* x, const void* Wpacked, const void* scales, int64_t group,
                             void* y, int64_t M, int64_t N, int64_t K, void* stream);

/*
 * tl_ternary_gemm_grouped for the other two weight forms: several independent products in one
 * call, enqueued in as few kernel launches as possible (the launch costs as much as streaming
 * several megabytes, and the paper's kernel benchmark is quoted on all linears of a block,
 * App. G).  Jobs must not alias each other's outputs; `jobs` is host memory, read before the
 * call returns; each job has the contract of the single call it stands for.
 *
 * tl_ternary_gemm_1p6_grouped: weights in the 1.6-bit layout (Sec. 3.2), all jobs in the same
 * byte code: `format` is TL_FMT_1P6BIT (tl_pack_1p6bit) or TL_FMT_1P6BIT_FX (tl_pack_1p6bit_fx),
 * anything else is TL_ERR_VALUE.  Jobs with K % 8 == 0 and K <= 4480 share launches (32 blocks
 * of 16 activation rows per launch); the others run as tl_ternary_gemm_1p6 / _fx would run them.
 */
tl_status tl_ternary_gemm_1p6_grouped(const tl_gemm_job* jobs, int64_t count, tl_format format,
                                      void* stream);

/*
 * tl_ternary_gemm_gs_grouped: 2-bit weights with per-group scales (Sec. 3.3; App. G), one group
 * size per job.  Jobs that tl_ternary_gemm_gs would run in the weight-streaming kernel share
 * launches (groups that are multiples of 256 weights among themselves, odd multiples of 128
 * among themselves); the others run one by one.
 */
typedef struct tl_gemm_gs_job {
    const void* x;            /* device, fp16 [M][K]                         */
    const void* Wpacked;      /* device, TL_FMT_2BIT                         */
    const void* scales;       /* device, fp16 [ceil(K / group)][N]           */
    void* y;                  /* device, fp16 [M][N]                         */
    int64_t M, N, K;
    int64_t group;            /* weights per scale along K, multiple of 16   */
} tl_gemm_gs_job;

tl_status tl_ternary_gemm_gs_grouped(const tl_gemm_gs_job* jobs, int64_t count, void* stream);

/*
 * Bandwidth calibration: a plain streaming copy dst[i] = src[i] of `bytes` bytes
 * (multiple of 16, both device pointers 16-byte aligned).  Not part of the
 * method; it gives the HBM counters and timers a kernel of known traffic.
 */
tl_status tl_probe_copy(void* dst, const void* src, size_t bytes, void* stream);

/*
 * Bandwidth ceiling: a streaming read of `bytes` bytes (multiple of 16, `src` a device
 * pointer, 16-byte aligned) that does nothing with them -- one launch, as many workgroups as
 * the buffer has 16 KB pieces.  No kernel that streams a weight matrix of that size once per
 * launch (Sec. 3.3: the memory-bound regime) can finish sooner; the benchmark times it beside
 * the GEMM kernels.  `sink` is a device pointer to 4 writable bytes, 4-byte aligned, written
 * only if the fold of all words read equals one particular value (it keeps the loads alive).
 * Not part of the method.
 */
tl_status tl_probe_read(const void* src, size_t bytes, void* sink, void* stream);

/*
 * Matrix-pipe ceiling for the large-batch regime (Sec. 3.3: beyond the critical batch the product
 * is compute-bound; App. G: the dequantised weights feed the matrix units): a kernel whose waves
 * do nothing but fp16 matrix instructions (v_mfma_f32_32x32x16_f16, 8 independent accumulators
 * per wave, two waves per SIMD of a 256-CU device) for `iters` rounds.  The operands are real data,
 * since what the chip sustains depends on it: activations read from `x` (device, fp16, x_elems >= 1
 * of them, reused cyclically) against ternary weights decoded to -1 / 0 / +1 from `Wpacked`
 * (device, 2-bit words, w_words >= 1).  `*flops` (host, may be NULL) receives the floating-point
 * operations of the launch; `sink` is a device pointer to 4 writable bytes (written only if the
 * fold of all sums equals one particular value).  Not part of the method: the benchmark times it
 * beside the large-M kernel.
 */
tl_status tl_probe_mfma(const void* x, int64_t x_elems, const void* Wpacked, int64_t w_words, int64_t iters,
                        void* sink, double* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TL_H_ */
