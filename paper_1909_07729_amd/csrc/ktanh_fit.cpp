// Host side of libktanh: the offline parameter optimisation of Section 2.4 for BFloat16 inputs.
//
// For every interval of inputs (fixed low exponent bits and leading mantissa bits):
//   Step 1  evaluate TanH on the interval's inputs, split each value into exponent and mantissa;
//   Step 2  choose one output exponent for the whole interval: the candidate, among the exponents
//           that occur, with the least squared error once the other values' mantissas are pinned
//           to 0 (below the candidate's binade) or 2^q - 1 (above it);
//   Step 3  choose the shift r and offset b that minimise eq. (1), sum (M^_i - (m_i / 2^r + b))^2,
//           with b rounded from the least-squares solution and clamped to [b_min, b_max] (eq. (2))
//           so that shift-and-add can neither underflow nor overflow the 7-bit mantissa.
// Mantissas of TanH stay real numbers and m_i / 2^r is a real division throughout: with these two
// readings the fit returns exactly the 32 triples the paper prints in Table 1.
#include <cmath>
#include <limits>
#include <vector>

#include "ktanh.h"

namespace {

constexpr int kMantissaBits = 7;   // p: BFloat16 input mantissa
constexpr int kOutMantissaBits = 7;  // q: BFloat16 output mantissa

struct Sample {
    double m;        // input mantissa as an integer value
    double y;        // TanH of the input
    int exponent;    // biased exponent of y
    double mantissa; // real-valued mantissa of y in units of 2^-q
};

struct Fit {
    int E, r, b;
};

// Inputs of interval t when `index_bits` leading mantissa bits take part in the index.
std::vector<Sample> interval_samples(int t, int index_bits)
{
    const int count = 1 << (kMantissaBits - index_bits);
    const int mantissa_idx_val = t & ((1 << index_bits) - 1);
    const int low_exp_bits = t >> index_bits;
    int input_exponent = 125;
    while ((input_exponent & 3) != low_exp_bits) ++input_exponent;  // 125..128 tile [0.25, 4)

    std::vector<Sample> out;
    for (int k = 0; k < count; ++k) {
        Sample s;
        s.m = mantissa_idx_val * count + k;
        const double x = std::ldexp(1.0 + s.m / (1 << kMantissaBits), input_exponent - 127);
        s.y = std::tanh(x);
        const int unbiased = std::ilogb(s.y);
        s.exponent = unbiased + 127;
        s.mantissa = (std::ldexp(s.y, -unbiased) - 1.0) * (1 << kOutMantissaBits);
        out.push_back(s);
    }
    return out;
}

double pinned_mantissa(const Sample &s, int E)
{
    if (s.exponent == E) return s.mantissa;
    return E > s.exponent ? 0.0 : double((1 << kOutMantissaBits) - 1);
}

// offsets_add_only: the ablation of Section 3, which sets b_min = 0.
Fit fit_interval(int t, int index_bits, bool offsets_add_only = false)
{
    const std::vector<Sample> pts = interval_samples(t, index_bits);
    const int mantissa_idx_val = t & ((1 << index_bits) - 1);
    const int per = (int)pts.size();

    // Step 2
    int E = pts.front().exponent;
    double least = std::numeric_limits<double>::infinity();
    for (const Sample &cand : pts) {
        double err = 0.0;
        for (const Sample &s : pts) {
            const double yhat = std::ldexp(1.0 + pinned_mantissa(s, cand.exponent) / (1 << kOutMantissaBits),
                                           cand.exponent - 127);
            err += (s.y - yhat) * (s.y - yhat);
        }
        if (err < least) { least = err; E = cand.exponent; }
    }

    // Step 3
    Fit best{E, 0, 0};
    double best_obj = std::numeric_limits<double>::infinity();
    for (int r = 0; r <= kMantissaBits; ++r) {
        const double step = std::ldexp(1.0, -r);  // 1 / 2^r
        double residual = 0.0;
        for (const Sample &s : pts) residual += pinned_mantissa(s, E) - s.m * step;
        long b = std::lround(std::floor(residual / per + 0.5));
        const long last_m = (long)(mantissa_idx_val + 1) * per - 1;
        const long b_max = (1L << kMantissaBits) - 1 - (last_m >> r);
        const int width = kMantissaBits - index_bits - r;
        const long b_min = offsets_add_only ? 0L : -(long)mantissa_idx_val * (width >= 0 ? (1L << width) : 0L);
        if (b < b_min) b = b_min;
        if (b > b_max) b = b_max;
        double obj = 0.0;
        for (const Sample &s : pts) {
            const double d = pinned_mantissa(s, E) - (s.m * step + (double)b);
            obj += d * d;
        }
        if (obj < best_obj) { best_obj = obj; best.r = r; best.b = (int)b; }
    }
    return best;
}

}  // namespace

extern "C" ktanh_status_t ktanh_fit_lut(ktanh_lut_t *out)
{
    if (out == nullptr) return KT_ERR_NULL;
    for (int t = 0; t < KTANH_INTERVALS; ++t) {
        const Fit f = fit_interval(t, 3);
        out->E[t] = (uint8_t)f.E;
        out->r[t] = (uint8_t)f.r;
        out->b[t] = (int8_t)f.b;
    }
    return KT_OK;
}

extern "C" ktanh_status_t ktanh_fit_lut_bmin0(ktanh_lut_t *out)
{
    if (out == nullptr) return KT_ERR_NULL;
    for (int t = 0; t < KTANH_INTERVALS; ++t) {
        const Fit f = fit_interval(t, 3, true);
        out->E[t] = (uint8_t)f.E;
        out->r[t] = (uint8_t)f.r;
        out->b[t] = (int8_t)f.b;
    }
    return KT_OK;
}

extern "C" ktanh_status_t ktanh_fit_lut64(ktanh_lut64_t *out)
{
    if (out == nullptr) return KT_ERR_NULL;
    for (int t = 0; t < KTANH_INTERVALS64; ++t) {
        const Fit f = fit_interval(t, 4);
        out->E[t] = (uint8_t)f.E;
        out->r[t] = (uint8_t)f.r;
        out->b[t] = (int8_t)f.b;
    }
    return KT_OK;
}
