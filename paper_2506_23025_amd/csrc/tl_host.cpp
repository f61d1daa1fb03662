// Host side of the ternary-linear library: geometry, packers and the host decoders.
// Pure C++ (no HIP calls); compiled into libtl.so together with the kernels.
#include "tl.h"

#include <cmath>
#include <cstring>

namespace {

constexpr int kTritsPerByte = 5;

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

inline bool shape_ok(int64_t N, int64_t K) {
    return N >= 1 && K >= 1 && N < (int64_t(1) << 40) && K < (int64_t(1) << 40);
}

// digit = w + 1 for w in {-1,0,1}; anything else maps to a value > 2.
inline unsigned digit_of(int8_t w) { return static_cast<unsigned>(static_cast<uint8_t>(w + 1)); }

// Base-3 byte -> its five digits, least significant first (digits of v mod 243 for v > 242).
struct Base3Table {
    uint8_t d[256][kTritsPerByte];
    Base3Table() {
        for (int v = 0; v < 256; ++v) {
            int r = v % 243;
            for (int i = 0; i < kTritsPerByte; ++i) { d[v][i] = static_cast<uint8_t>(r % 3); r /= 3; }
        }
    }
};

const Base3Table& base3_table() {
    static const Base3Table t;
    return t;
}

}  // namespace

extern "C" {

const char* tl_status_str(tl_status s) {
    switch (s) {
        case TL_OK: return "ok";
        case TL_ERR_NULL: return "null pointer";
        case TL_ERR_SHAPE: return "bad shape";
        case TL_ERR_VALUE: return "value outside the ternary code";
        case TL_ERR_ALIGN: return "pointer not 16-byte aligned";
        case TL_ERR_UNSUPPORTED: return "unsupported format, path or shape";
        case TL_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

size_t tl_row_stride_bytes(tl_format fmt, int64_t K) {
    if (K < 1 || K >= (int64_t(1) << 40)) return 0;
    switch (fmt) {
        case TL_FMT_2BIT: return static_cast<size_t>(4 * ceil_div(K, 16));
        case TL_FMT_1P6BIT:
        case TL_FMT_1P6BIT_FX: return static_cast<size_t>(16 * ceil_div(ceil_div(K, kTritsPerByte), 16));
        default: return 0;                       // an unknown format
    }
}

size_t tl_packed_bytes(tl_format fmt, int64_t N, int64_t K) {
    if (!shape_ok(N, K)) return 0;
    return static_cast<size_t>(N) * tl_row_stride_bytes(fmt, K);
}

// Sec. 3.1 with k = 16: the word is built from its top digit down (Horner in base 4),
// which leaves weight 16i+j in bits [2j+1:2j].
namespace {

// fp64 -> fp16 bits, round to nearest even; subnormals kept, overflow to infinity.
uint16_t double_to_half_bits(double v) {
    const uint16_t sign = std::signbit(v) ? 0x8000u : 0u;
    const double a = std::fabs(v);
    if (std::isnan(a)) return static_cast<uint16_t>(sign | 0x7E00u);
    if (a >= 65520.0) return static_cast<uint16_t>(sign | 0x7C00u);
    int e = 0;
    (void)std::frexp(a, &e);                        // a = f * 2^e, f in [0.5, 1)
    e -= 1;                                         // a in [2^e, 2^(e+1))
    if (a == 0.0 || e < -14) {                      // subnormal range: units of 2^-24
        const double q = std::nearbyint(std::ldexp(a, 24));
        return static_cast<uint16_t>(sign | static_cast<uint16_t>(q));   // q = 1024 is the least normal
    }
    double m = std::nearbyint(std::ldexp(a, 10 - e));                    // in [1024, 2048]
    if (m >= 2048.0) { m = 1024.0; e += 1; }
    if (e > 15) return static_cast<uint16_t>(sign | 0x7C00u);
    return static_cast<uint16_t>(sign | ((e + 15) << 10) | (static_cast<int>(m) - 1024));
}

}  // namespace

// App. B "Forward Pass": gamma = eps + mean |W|, What = round(clip(W / gamma, -1, 1)).
tl_status tl_quantize(const float* W, int64_t N, int64_t K, double eps, int8_t* What,
                      double* gamma, uint16_t* gamma_fp16_bits) {
    if (!W || !What) return TL_ERR_NULL;
    if (!shape_ok(N, K)) return TL_ERR_SHAPE;
    if (!(eps >= 0.0) || !std::isfinite(eps)) return TL_ERR_VALUE;
    const int64_t count = N * K;
    // sum of |W| in fp64 with a running compensation (Neumaier), so that the result does not
    // depend on the order more than in its last bit
    double sum = 0.0, comp = 0.0;
    bool bad = false;
    for (int64_t i = 0; i < count; ++i) {
        const double a = std::fabs(static_cast<double>(W[i]));
        bad |= !std::isfinite(a);
        const double t = sum + a;
        comp += (sum >= a) ? (sum - t) + a : (a - t) + sum;
        sum = t;
    }
    if (bad) return TL_ERR_VALUE;
    const double g = eps + (sum + comp) / static_cast<double>(count);
    if (gamma) *gamma = g;
    if (gamma_fp16_bits) *gamma_fp16_bits = double_to_half_bits(g);
    for (int64_t i = 0; i < count; ++i) {
        double q = (g > 0.0) ? static_cast<double>(W[i]) / g : 0.0;
        q = q < -1.0 ? -1.0 : (q > 1.0 ? 1.0 : q);
        What[i] = static_cast<int8_t>(std::nearbyint(q));              // half to even
    }
    return TL_OK;
}

tl_status tl_pack_2bit(const int8_t* W, int64_t N, int64_t K, uint32_t* out) {
    if (!W || !out) return TL_ERR_NULL;
    if (!shape_ok(N, K)) return TL_ERR_SHAPE;
    const int64_t words = ceil_div(K, 16);
    unsigned bad = 0;
    for (int64_t n = 0; n < N; ++n) {
        const int8_t* row = W + n * K;
        uint32_t* dst = out + n * words;
        for (int64_t i = 0; i < words; ++i) {
            const int64_t base = 16 * i;
            const int len = static_cast<int>(K - base < 16 ? K - base : 16);
            uint32_t word = 0;
            for (int j = 15; j >= 0; --j) {
                const unsigned dgt = (j < len) ? digit_of(row[base + j]) : 1u;
                bad |= (dgt > 2u);
                word = (word << 2) | (dgt & 3u);
            }
            dst[i] = word;
        }
    }
    return bad ? TL_ERR_VALUE : TL_OK;
}

// Plain base-3 byte, digit i of the byte = weight 5b+i (Horner from the top digit).
tl_status tl_pack_1p6bit(const int8_t* W, int64_t N, int64_t K, uint8_t* out) {
    if (!W || !out) return TL_ERR_NULL;
    if (!shape_ok(N, K)) return TL_ERR_SHAPE;
    const int64_t stride = static_cast<int64_t>(tl_row_stride_bytes(TL_FMT_1P6BIT, K));
    const int64_t nbytes = ceil_div(K, kTritsPerByte);
    unsigned bad = 0;
    for (int64_t n = 0; n < N; ++n) {
        const int8_t* row = W + n * K;
        uint8_t* dst = out + n * stride;
        for (int64_t b = 0; b < nbytes; ++b) {
            const int64_t base = kTritsPerByte * b;
            unsigned v = 0;
            for (int i = kTritsPerByte - 1; i >= 0; --i) {
                const unsigned dgt = (base + i < K) ? digit_of(row[base + i]) : 1u;
                bad |= (dgt > 2u);
                v = v * 3u + (dgt > 2u ? 0u : dgt);
            }
            dst[b] = static_cast<uint8_t>(v);
        }
        std::memset(dst + nbytes, 0, static_cast<size_t>(stride - nbytes));
    }
    return bad ? TL_ERR_VALUE : TL_OK;
}

// Sec. 3.2 / App. E with k = 5, p = 8: digits big-endian, byte = floor((256 Nval + 242) / 243).
tl_status tl_pack_1p6bit_fx(const int8_t* W, int64_t N, int64_t K, uint8_t* out) {
    if (!W || !out) return TL_ERR_NULL;
    if (!shape_ok(N, K)) return TL_ERR_SHAPE;
    const int64_t stride = static_cast<int64_t>(tl_row_stride_bytes(TL_FMT_1P6BIT, K));
    const int64_t nbytes = ceil_div(K, kTritsPerByte);
    unsigned bad = 0;
    for (int64_t n = 0; n < N; ++n) {
        const int8_t* row = W + n * K;
        uint8_t* dst = out + n * stride;
        for (int64_t b = 0; b < nbytes; ++b) {
            const int64_t base = kTritsPerByte * b;
            unsigned nval = 0;
            for (int j = 0; j < kTritsPerByte; ++j) {
                const unsigned dgt = (base + j < K) ? digit_of(row[base + j]) : 1u;
                bad |= (dgt > 2u);
                nval = nval * 3u + (dgt > 2u ? 0u : dgt);
            }
            dst[b] = static_cast<uint8_t>((nval * 256u + 242u) / 243u);
        }
        std::memset(dst + nbytes, 0, static_cast<size_t>(stride - nbytes));
    }
    return bad ? TL_ERR_VALUE : TL_OK;
}

// Decode of the fixed-point code: b = ceil(256 V / 243) is inverted by V = floor(243 b / 256),
// and V's base-3 digits, most significant first, are the weights + 1.  (App. F, Alg. 1 peels the
// same digits off with multiplications by 3; the tests hold this decode against it.)
tl_status tl_unpack_1p6bit_fx(const uint8_t* packed, int64_t N, int64_t K, int8_t* W_out) {
    if (!packed || !W_out) return TL_ERR_NULL;
    if (!shape_ok(N, K)) return TL_ERR_SHAPE;
    const int64_t stride = static_cast<int64_t>(tl_row_stride_bytes(TL_FMT_1P6BIT, K));
    static const unsigned kPow3[kTritsPerByte] = {81u, 27u, 9u, 3u, 1u};
    for (int64_t n = 0; n < N; ++n) {
        const uint8_t* src = packed + n * stride;
        int8_t* row = W_out + n * K;
        for (int64_t base = 0; base < K; base += kTritsPerByte) {
            const unsigned value = (243u * src[base / kTritsPerByte]) >> 8;
            for (int i = 0; i < kTritsPerByte && base + i < K; ++i)
                row[base + i] = static_cast<int8_t>(static_cast<int>((value / kPow3[i]) % 3u) - 1);
        }
    }
    return TL_OK;
}

tl_status tl_unpack(tl_format fmt, const void* packed, int64_t N, int64_t K, int8_t* W_out) {
    if (!packed || !W_out) return TL_ERR_NULL;
    if (!shape_ok(N, K)) return TL_ERR_SHAPE;
    unsigned bad = 0;
    if (fmt == TL_FMT_2BIT) {
        const int64_t words = ceil_div(K, 16);
        const uint32_t* src = static_cast<const uint32_t*>(packed);
        for (int64_t n = 0; n < N; ++n) {
            int8_t* row = W_out + n * K;
            for (int64_t i = 0; i < words; ++i) {
                uint32_t word = src[n * words + i];
                const int64_t base = 16 * i;
                const int len = static_cast<int>(K - base < 16 ? K - base : 16);
                for (int j = 0; j < len; ++j, word >>= 2) {
                    const unsigned dgt = word & 3u;
                    bad |= (dgt == 3u);
                    row[base + j] = static_cast<int8_t>(static_cast<int>(dgt) - 1);
                }
            }
        }
        return bad ? TL_ERR_VALUE : TL_OK;
    }
    if (fmt == TL_FMT_1P6BIT) {
        const Base3Table& T = base3_table();
        const int64_t stride = static_cast<int64_t>(tl_row_stride_bytes(fmt, K));
        const uint8_t* src = static_cast<const uint8_t*>(packed);
        for (int64_t n = 0; n < N; ++n) {
            int8_t* row = W_out + n * K;
            for (int64_t base = 0; base < K; base += kTritsPerByte) {
                const uint8_t v = src[n * stride + base / kTritsPerByte];
                bad |= (v > 242u);
                for (int i = 0; i < kTritsPerByte && base + i < K; ++i)
                    row[base + i] = static_cast<int8_t>(static_cast<int>(T.d[v][i]) - 1);
            }
        }
        return bad ? TL_ERR_VALUE : TL_OK;
    }
    if (fmt == TL_FMT_1P6BIT_FX)
        return tl_unpack_1p6bit_fx(static_cast<const uint8_t*>(packed), N, K, W_out);
    return TL_ERR_UNSUPPORTED;
}

}  // extern "C"
