#include "common.h"

#include <cstring>

namespace apnn {

char *error_buffer()
{
    static thread_local char buf[512] = {0};
    return buf;
}

void clear_error() { error_buffer()[0] = 0; }

int fail(apnn_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(error_buffer(), 512, fmt, ap);
    va_end(ap);
    return static_cast<int>(st);
}

int check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(APNN_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
    return APNN_OK;
}

int check_bits_enc(const char *who, const char *name, int bits, apnn_encoding enc)
{
    if (bits < 1 || bits > 8) return fail(APNN_ERR_UNSUPPORTED, "%s: %s bits = %d, supported 1..8", who, name, bits);
    if (enc != APNN_ENC_UNSIGNED && enc != APNN_ENC_PM1)
        return fail(APNN_ERR_INVALID_ARG, "%s: unknown encoding %d for %s", who, static_cast<int>(enc), name);
    if (enc == APNN_ENC_PM1 && bits != 1)
        return fail(APNN_ERR_UNSUPPORTED, "%s: the -1/+1 encoding is defined for 1-bit %s only (got %d bits)", who, name, bits);
    return APNN_OK;
}

int check_int32_range(const char *who, int64_t K, int p, int q)
{
    const int64_t worst = K * ((int64_t(1) << p) - 1) * ((int64_t(1) << q) - 1);
    if (worst >= (int64_t(1) << 31))
        return fail(APNN_ERR_OVERFLOW, "%s: K(2^p-1)(2^q-1) = %lld does not fit int32", who, static_cast<long long>(worst));
    return APNN_OK;
}

}  // namespace apnn

extern "C" const char *apnn_last_error(void) { return apnn::error_buffer(); }

extern "C" int64_t apnn_row_words(int64_t K)
{
    if (K < 0) return 0;
    return apnn::round_up(apnn::ceil_div(K, 32), 4);
}

extern "C" size_t apnn_packed_words(int64_t rows, int64_t K, int bits)
{
    if (rows < 0 || K < 0 || bits < 1 || bits > 8) return 0;
    return static_cast<size_t>(rows) * static_cast<size_t>(bits) * static_cast<size_t>(apnn_row_words(K));
}

extern "C" size_t apnn_fmap_words(int64_t pixels, int64_t C, int bits)
{
    if (pixels < 0 || C < 0 || bits < 1 || bits > 8) return 0;
    return static_cast<size_t>(pixels) * static_cast<size_t>(bits) * static_cast<size_t>(apnn::ceil_div(C, 32));
}

extern "C" int apnn_fold_bn(const double *gamma, const double *beta, const double *mean, const double *var,
                            double eps, double zero, double step, int64_t C, float *scale, float *bias)
{
    apnn::clear_error();
    if (!gamma || !beta || !mean || !var || !scale || !bias || C < 0)
        return apnn::fail(APNN_ERR_INVALID_ARG, "apnn_fold_bn: null pointer or negative C");
    if (!(step > 0.0)) return apnn::fail(APNN_ERR_INVALID_ARG, "apnn_fold_bn: step must be > 0");
    for (int64_t c = 0; c < C; ++c) {
        if (!(var[c] + eps > 0.0)) return apnn::fail(APNN_ERR_INVALID_ARG, "apnn_fold_bn: var+eps <= 0 at channel %lld", (long long)c);
        const double sd = __builtin_sqrt(var[c] + eps);
        scale[c] = static_cast<float>(gamma[c] / (sd * step));
        bias[c] = static_cast<float>((beta[c] - mean[c] * gamma[c] / sd - zero) / step);
    }
    return APNN_OK;
}
