/*
 * ternary_oracle.c -- TEST INFRASTRUCTURE, not a product path.
 *
 * A plain, slow, obviously-correct CPU statement of what the ternary linear
 * layer of Spectra-1.1 (arXiv 2506.23025) computes, written from the paper's
 * definitions.  Only tests, the smoke check and the bench's cpu_baseline leg
 * may call it.  It shares no code, header, table or constant with the HIP
 * library; nothing here is tuned, blocked, fused or reordered.
 *
 * What is here, and the passage each piece follows:
 *   orc_pack2 / orc_unpack2         Sec. 3.1  packing P and unpacking U, k digits
 *                                   per block (the GPU format uses k = 16)
 *   orc_pack_fx / orc_unpack_fx_div Sec. 3.2 / App. E  fixed-point base-3 code
 *                                   with parameters (k, p) and its division decode
 *   orc_unpack_fx_alg1              App. F, Alg. 1  multiply-by-3 digit extraction
 *   orc_pack3le / orc_unpack3le     the unscaled little-endian base-3 byte
 *                                   sum_i (w_i+1) 3^i used by the 1.6-bit GPU format
 *   orc_half_to_double              IEEE binary16 -> double, exact
 *   orc_gemm                        App. B "Inference": Y = X (gamma What)^T,
 *                                   double accumulation, k ascending
 *   orc_gemm_fixed                  the same sum in exact 2^-24 fixed point (int64)
 *
 * Pins (tests/test_oracle_*.py): closed-form words, exhaustive 3^5 / 3^8 block
 * enumeration, Theorem 1 both directions, Alg. 1 == division decode, brute-force
 * hand sums, numpy fp64 matmul, algebraic identities.  Parity unpinned: none.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------- 2-bit --- */

/* Sec. 3.1: d' = d + 1; block i is sum_j d'_{ki+j} 2^{2j}; a short last block is
 * filled with d = 0, i.e. digit 1.  n digits -> ceil(n/k) blocks, k <= 32.
 * Returns -1 if a digit is not in {-1,0,1}. */
int orc_pack2(const int8_t* d, int64_t n, int k, uint64_t* blocks)
{
    int64_t m = (n + k - 1) / k;
    for (int64_t i = 0; i < m; ++i) {
        uint64_t b = 0;
        for (int j = 0; j < k; ++j) {
            int64_t idx = (int64_t)k * i + j;
            int dj = (idx < n) ? d[idx] : 0;
            if (dj < -1 || dj > 1) return -1;
            uint64_t dp = (uint64_t)(dj + 1);
            b += dp << (2 * j);
        }
        blocks[i] = b;
    }
    return 0;
}

/* Sec. 3.1: d'_{ki+j} = (b_i >> 2j) & 3 ; d = d' - 1.  Returns -1 on a digit 3. */
int orc_unpack2(const uint64_t* blocks, int64_t n, int k, int8_t* d)
{
    for (int64_t idx = 0; idx < n; ++idx) {
        int64_t i = idx / k;
        int j = (int)(idx % k);
        int dp = (int)((blocks[i] >> (2 * j)) & 0x03);
        if (dp == 3) return -1;
        d[idx] = (int8_t)(dp - 1);
    }
    return 0;
}

/* Matrix form used by the GPU format: W int8 [N][K], one row = ceil(K/16) uint32. */
int orc_pack2_matrix(const int8_t* W, int64_t N, int64_t K, uint32_t* out)
{
    int64_t words = (K + 15) / 16;
    uint64_t blk[1];
    for (int64_t n = 0; n < N; ++n)
        for (int64_t i = 0; i < words; ++i) {
            int64_t left = K - 16 * i;
            int64_t len = left < 16 ? left : 16;
            if (orc_pack2(W + n * K + 16 * i, len, 16, blk) != 0) return -1;
            out[n * words + i] = (uint32_t)blk[0];
        }
    return 0;
}

int orc_unpack2_matrix(const uint32_t* packed, int64_t N, int64_t K, int8_t* W)
{
    int64_t words = (K + 15) / 16;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            uint32_t b = packed[n * words + k / 16];
            int dp = (int)((b >> (2 * (k % 16))) & 0x03);
            if (dp == 3) return -1;
            W[n * K + k] = (int8_t)(dp - 1);
        }
    return 0;
}

/* ------------------------------------------- fixed-point base-3 (k, p) --- */

static int64_t ipow(int64_t b, int e) { int64_t r = 1; while (e-- > 0) r *= b; return r; }

/* Mathematical floor of a / b for b > 0 (C division truncates toward zero). */
static int64_t floor_div(int64_t a, int64_t b)
{
    int64_t q = a / b;
    if (a % b != 0 && a < 0) --q;
    return q;
}

/* Sec. 3.2 / App. E: Nval = sum_j d'_j 3^{k-1-j};  b = floor((Nval 2^p + 3^k - 1) / 3^k).
 * One block of exactly k digits (the caller pads a short block with d = 0). */
int64_t orc_pack_fx_block(const int8_t* d, int k, int p)
{
    int64_t Nval = 0;
    for (int j = 0; j < k; ++j) {
        if (d[j] < -1 || d[j] > 1) return -1;
        Nval += (int64_t)(d[j] + 1) * ipow(3, k - 1 - j);
    }
    int64_t t = ipow(3, k);
    return (Nval * ((int64_t)1 << p) + (t - 1)) / t;
}

/* App. E: x = floor((b 3^k - (3^k - 1) + (2^p - 1)) / 2^p);  d'_j = floor(x / 3^{k-1-j}) mod 3. */
void orc_unpack_fx_div_block(int64_t b, int k, int p, int8_t* d)
{
    int64_t t = ipow(3, k);
    int64_t two_p = (int64_t)1 << p;
    int64_t num = b * t - (t - 1) + (two_p - 1);
    int64_t x = floor_div(num, two_p);
    for (int j = 0; j < k; ++j) {
        int64_t q = x / ipow(3, k - 1 - j);
        d[j] = (int8_t)((q % 3) - 1);
    }
}

/* App. F, Alg. 1 (k = 5, p = 8): b_0 = b; d'_i = (3 b_i) >> 8; b_{i+1} = (3 b_i) & 0xFF. */
void orc_unpack_fx_alg1_block(int b, int8_t* d)
{
    int cur = b;
    for (int i = 0; i < 5; ++i) {
        int prod = cur * 3;
        d[i] = (int8_t)((prod >> 8) - 1);
        cur = prod & 0xFF;
    }
}

/* ------------------------------------ plain little-endian base-3 byte --- */

static int64_t stride3(int64_t K) { int64_t nb = (K + 4) / 5; return (nb + 15) / 16 * 16; }

int64_t orc_stride3le(int64_t K) { return stride3(K); }

int orc_pack3le_matrix(const int8_t* W, int64_t N, int64_t K, uint8_t* out)
{
    int64_t stride = stride3(K);
    for (int64_t n = 0; n < N; ++n) {
        memset(out + n * stride, 0, (size_t)stride);
        for (int64_t b = 0; b < (K + 4) / 5; ++b) {
            int v = 0, pw = 1;
            for (int i = 0; i < 5; ++i) {
                int64_t k = 5 * b + i;
                int w = (k < K) ? W[n * K + k] : 0;
                if (w < -1 || w > 1) return -1;
                v += (w + 1) * pw;
                pw *= 3;
            }
            out[n * stride + b] = (uint8_t)v;
        }
    }
    return 0;
}

int orc_unpack3le_matrix(const uint8_t* packed, int64_t N, int64_t K, int8_t* W)
{
    int64_t stride = stride3(K);
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            int v = packed[n * stride + k / 5];
            if (v > 242) return -1;
            int i = (int)(k % 5);
            for (int s = 0; s < i; ++s) v /= 3;
            W[n * K + k] = (int8_t)(v % 3 - 1);
        }
    return 0;
}

/* ------------------------------------------------------------- numbers --- */

/* IEEE 754 binary16 -> double: sign, 5-bit exponent (bias 15), 10-bit fraction. */
double orc_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int f = h & 0x3FF;
    double v;
    if (e == 0)       v = ldexp((double)f, -24);                 /* zero / subnormal   */
    else if (e == 31) v = (f == 0) ? INFINITY : NAN;
    else              v = ldexp(1.0 + (double)f / 1024.0, e - 15);
    return sign ? -v : v;
}

/* ---------------------------------------------------------------- GEMM --- */

/* App. B "Inference": Wtilde = gamma What;  Y = X Wtilde^T.
 * S[m][n] = sum_{k=0}^{K-1} x[m][k] * w[n][k] in double, k ascending;
 * y[m][n] = gamma * S[m][n], kept in double (the caller rounds if it wants fp16).
 * x: fp16 bits [M][K]; W: int8 [N][K]; y: double [M][N].
 * The only parallelism is an outer split of n over the host threads. */
void orc_gemm(const uint16_t* x, const int8_t* W, uint16_t gamma_bits, double* y,
              int64_t M, int64_t N, int64_t K)
{
    double gamma = orc_half_to_double(gamma_bits);
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t m = 0; m < M; ++m) {
            double S = 0.0;
            for (int64_t k = 0; k < K; ++k)
                S += orc_half_to_double(x[m * K + k]) * (double)W[n * K + k];
            y[m * N + n] = gamma * S;
        }
}

/* The oracle proper for packed input: unpack (Sec. 3.1), then orc_gemm.
 * scratch: int8 [N][K] supplied by the caller.  Returns -1 on an invalid code. */
int orc_gemm_packed2(const uint16_t* x, const uint32_t* Wp, uint16_t gamma_bits, double* y,
                     int64_t M, int64_t N, int64_t K, int8_t* scratch)
{
    if (orc_unpack2_matrix(Wp, N, K, scratch) != 0) return -1;
    orc_gemm(x, scratch, gamma_bits, y, M, N, K);
    return 0;
}

int orc_gemm_packed3le(const uint16_t* x, const uint8_t* Wp, uint16_t gamma_bits, double* y,
                       int64_t M, int64_t N, int64_t K, int8_t* scratch)
{
    if (orc_unpack3le_matrix(Wp, N, K, scratch) != 0) return -1;
    orc_gemm(x, scratch, gamma_bits, y, M, N, K);
    return 0;
}

/* Second, independent form of the same sum.  Every finite fp16 is an integer
 * multiple of 2^-24, so S 2^24 = sum_k (x_k 2^24) w_k is an exact integer sum:
 * no rounding and no dependence on order (|x| <= 65504 and K < 2^22 keep it
 * inside int64).  S24[m][n] receives that integer.  Returns -1 on inf/NaN in x. */
int orc_gemm_fixed(const uint16_t* x, const int8_t* W, int64_t* S24,
                   int64_t M, int64_t N, int64_t K)
{
    for (int64_t i = 0; i < M * K; ++i)
        if (((x[i] >> 10) & 0x1F) == 31) return -1;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int64_t acc = 0;
            for (int64_t k = K - 1; k >= 0; --k) {         /* descending on purpose */
                uint16_t h = x[m * K + k];
                int e = (h >> 10) & 0x1F;
                int64_t f = h & 0x3FF;
                int64_t mag = (e == 0) ? f : ((f + 1024) << (e - 1));
                int64_t xv = (h & 0x8000) ? -mag : mag;
                acc += xv * (int64_t)W[n * K + k];
            }
            S24[m * N + n] = acc;
        }
    return 0;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
