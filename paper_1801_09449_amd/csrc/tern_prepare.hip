// Host-side model preparation (runs on the CPU, touches no device memory): turning trained float
// weights and batch-norm statistics into what the convolution kernels take -- ternary filter
// codes plus one scale per output channel (Eq. 4, or with a prescribed number of zeros per filter
// as in the remark after Eq. 9), and two integer cut points per output channel
// that reproduce the ternary activation (Eq. 6) applied after scale and batch-norm (section 2).
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <vector>

#include "tern.h"

namespace {

// Eq. 6 on y = a*acc + b, in double.
inline int code_of(double a, double b, int64_t acc)
{
    const double y = a * (double)acc + b;
    if (y > 0.5) return 1;
    if (std::fabs(y) <= 0.5) return 0;   // also false for NaN, which then falls to -1 like Eq. 6's "else"
    return -1;
}

}  // namespace

extern "C" {

int tern_ternarize_filters(const float* w, int32_t c_out, int64_t per_filter, int8_t* codes,
                           double* alpha)
{
    if (!w || !codes || !alpha) return TERN_ENULL;
    if (c_out <= 0 || per_filter <= 0) return TERN_ESHAPE;
    for (int32_t co = 0; co < c_out; ++co) {
        const float* row = w + (size_t)co * per_filter;
        int8_t* out = codes + (size_t)co * per_filter;
        double sum_abs = 0.0;
        for (int64_t i = 0; i < per_filter; ++i) sum_abs += std::fabs((double)row[i]);
        const double delta = 0.7 * sum_abs / (double)per_filter;
        double kept = 0.0;
        int64_t n_kept = 0;
        for (int64_t i = 0; i < per_filter; ++i) {
            const double v = (double)row[i];
            int8_t t = 0;
            if (v > delta) t = 1;
            else if (!(std::fabs(v) <= delta)) t = -1;
            out[i] = t;
            if (t != 0) { kept += std::fabs(v); ++n_kept; }
        }
        alpha[co] = n_kept ? kept / (double)n_kept : 0.0;
    }
    return TERN_OK;
}

int tern_ternarize_filters_sparse(const float* w, int32_t c_out, int64_t per_filter, int64_t zeros,
                                  int8_t* codes, double* alpha)
{
    if (!w || !codes || !alpha) return TERN_ENULL;
    if (c_out <= 0 || per_filter <= 0) return TERN_ESHAPE;
    if (zeros < 0 || zeros > per_filter) return TERN_EARG;
    std::vector<int64_t> order((size_t)per_filter);
    for (int32_t co = 0; co < c_out; ++co) {
        const float* row = w + (size_t)co * per_filter;
        int8_t* out = codes + (size_t)co * per_filter;
        for (int64_t i = 0; i < per_filter; ++i) order[(size_t)i] = i;
        // the `zeros` entries of smallest magnitude, equal magnitudes in index order: only the cut
        // matters, so a selection instead of a full sort
        const auto smaller = [row](int64_t a, int64_t b) {
            const float fa = std::fabs(row[a]), fb = std::fabs(row[b]);
            return fa < fb || (fa == fb && a < b);
        };
        if (zeros > 0 && zeros < per_filter)
            std::nth_element(order.begin(), order.begin() + zeros, order.end(), smaller);
        double kept = 0.0;
        int64_t n_kept = 0;
        for (int64_t r = 0; r < per_filter; ++r) {
            const int64_t i = order[(size_t)r];
            int8_t t = 0;
            if (r >= zeros) t = row[i] > 0.0f ? 1 : (row[i] < 0.0f ? -1 : 0);
            out[i] = t;
            if (t != 0) { kept += std::fabs((double)row[i]); ++n_kept; }
        }
        alpha[co] = n_kept ? kept / (double)n_kept : 0.0;
    }
    return TERN_OK;
}

int tern_digits_weights(const int8_t* w, int32_t c_out, int32_t c_in, int64_t taps, int8_t* w_out)
{
    if (!w || !w_out) return TERN_ENULL;
    if (c_out <= 0 || c_in <= 0 || taps <= 0) return TERN_ESHAPE;
    const int64_t wd = (c_in + 31) / 32;
    for (int32_t co = 0; co < c_out; ++co)
        for (int64_t c2 = 0; c2 < 64 * wd; ++c2) {
            const int64_t src = 32 * (c2 / 64) + c2 % 32;   // both words of a pair hold the same channels
            for (int64_t t = 0; t < taps; ++t)
                w_out[((size_t)co * 64 * wd + c2) * taps + t] =
                    src < c_in ? w[((size_t)co * c_in + src) * taps + t] : (int8_t)0;
        }
    return TERN_OK;
}

int tern_fold_thresholds(const double* scale, const double* shift, int32_t c, int32_t acc_bound,
                         int32_t* lo, int32_t* hi, uint8_t* negate)
{
    if (!scale || !shift || !lo || !hi || !negate) return TERN_ENULL;
    if (c <= 0) return TERN_ESHAPE;
    if (acc_bound < 1 || acc_bound >= (1 << 24)) return TERN_EARG;
    const int64_t B = acc_bound;
    for (int32_t ch = 0; ch < c; ++ch) {
        double a = scale[ch];
        const double b = shift[ch];
        if (!std::isfinite(a) || !std::isfinite(b)) return TERN_EARG;
        negate[ch] = a < 0.0 ? 1 : 0;
        if (a < 0.0) a = -a;   // the caller negates this filter: conv(-w) = -conv(w)
        // code(acc) is non-decreasing in acc for a >= 0.  hi = largest acc in [-B-1, B+1] whose
        // code is not +1 (or -B-1 if every acc in range gives +1); lo = smallest acc whose code
        // is not -1 (or B+1 if every acc gives -1).  Found by bisection on the double-precision
        // evaluation itself, so the integer rule agrees with it at every tie.
        int64_t lo_i, hi_i;
        {
            int64_t l = -B - 1, r = B + 1;            // invariant: code(l) < +1 or l == -B-1
            if (code_of(a, b, -B) == 1) hi_i = -B - 1;
            else {
                l = -B;                                // code(l) != +1
                if (code_of(a, b, B) != 1) hi_i = B + 1;
                else {
                    r = B;                             // code(r) == +1
                    while (r - l > 1) {
                        const int64_t m = l + (r - l) / 2;
                        if (code_of(a, b, m) == 1) r = m; else l = m;
                    }
                    hi_i = l;
                }
            }
        }
        {
            int64_t l, r;
            if (code_of(a, b, B) == -1) lo_i = B + 1;
            else {
                r = B;                                 // code(r) != -1
                if (code_of(a, b, -B) != -1) lo_i = -B - 1;
                else {
                    l = -B;                            // code(l) == -1
                    while (r - l > 1) {
                        const int64_t m = l + (r - l) / 2;
                        if (code_of(a, b, m) == -1) l = m; else r = m;
                    }
                    lo_i = r;
                }
            }
        }
        // lo_i == hi_i + 1 when no integer falls in the zero band (|scale| > 1): the -1 and +1
        // ranges are then adjacent and never overlap.
        lo[ch] = (int32_t)lo_i;
        hi[ch] = (int32_t)hi_i;
    }
    return TERN_OK;
}

int tern_fold_batchnorm(const double* alpha, const double* gamma, const double* beta,
                        const double* mean, const double* var, double eps, int32_t c,
                        int32_t acc_bound, int32_t* lo, int32_t* hi, uint8_t* negate)
{
    if (!alpha || !gamma || !beta || !mean || !var) return TERN_ENULL;
    if (c <= 0) return TERN_ESHAPE;
    if (!(eps >= 0.0)) return TERN_EARG;
    for (int32_t ch = 0; ch < c; ++ch) {
        if (!(var[ch] + eps > 0.0)) return TERN_EARG;
        const double inv = 1.0 / std::sqrt(var[ch] + eps);
        const double a = alpha[ch] * gamma[ch] * inv;
        const double b = beta[ch] - gamma[ch] * mean[ch] * inv;
        const int rc = tern_fold_thresholds(&a, &b, 1, acc_bound, lo + ch, hi + ch, negate + ch);
        if (rc != TERN_OK) return rc;
    }
    return TERN_OK;
}

int tern_fold_avgpool(const int8_t* w, int32_t c_out, int32_t c_in, int32_t kd, int32_t kh,
                      int32_t kw, const int32_t pool[3], int8_t* w_out)
{
    if (!w || !pool || !w_out) return TERN_ENULL;
    if (c_out <= 0 || c_in <= 0 || kd < 1 || kh < 1 || kw < 1) return TERN_ESHAPE;
    for (int a = 0; a < 3; ++a)
        if (pool[a] < 1 || pool[a] > 1024) return TERN_EARG;
    const int64_t fd = (int64_t)kd * pool[0], fh = (int64_t)kh * pool[1], fw = (int64_t)kw * pool[2];
    if (fd > 1024 || fh > 1024 || fw > 1024) return TERN_ESHAPE;
    const size_t filters = (size_t)c_out * (size_t)c_in;
    for (size_t f = 0; f < filters; ++f) {
        const int8_t* src = w + f * (size_t)kd * kh * kw;
        int8_t* dst = w_out + f * (size_t)(fd * fh * fw);
        for (int64_t a = 0; a < fd; ++a)
            for (int64_t b = 0; b < fh; ++b)
                for (int64_t c = 0; c < fw; ++c)
                    dst[(a * fh + b) * fw + c] =
                        src[((a / pool[0]) * kh + b / pool[1]) * kw + c / pool[2]];
    }
    return TERN_OK;
}

}  // extern "C"
