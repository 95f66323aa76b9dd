// Host side of libktanh: the paper's parameter table, its validation and its kernel-argument form.
#include "ktanh_pack.h"

#include <cmath>

namespace {

// Table 1 (optimised parameters for BFloat16 inputs), stored by integer index
// t = (E_i & 3) << 3 | (M_i >> 4); the paper prints the rows by descending input magnitude.
constexpr ktanh_lut_t kTable1 = {
    /* E */ {// t = 0..7  : |x| in [2, 4)
             126, 126, 126, 126, 126, 126, 126, 126,
             // t = 8..15 : [0.25, 0.5)
             125, 125, 125, 125, 125, 125, 125, 125,
             // t = 16..23: [0.5, 1)
             125, 126, 126, 126, 126, 126, 126, 126,
             // t = 24..31: [1, 2)
             126, 126, 126, 126, 126, 126, 126, 126},
    /* r */ {2, 4, 4, 4, 6, 6, 6, 6,
             1, 0, 0, 0, 0, 0, 0, 0,
             0, 1, 1, 1, 1, 1, 1, 1,
             0, 1, 1, 1, 2, 2, 2, 4},
    /* b */ {119, 122, 123, 123, 126, 126, 126, 126,
             1, -4, -6, -7, -10, -12, -15, -18,
             112, -4, -1, 2, 3, 4, 4, 4,
             65, 72, 73, 73, 88, 89, 89, 110},
};

}  // namespace

extern "C" const char *ktanh_status_string(ktanh_status_t status)
{
    switch (status) {
        case KT_OK: return "KT_OK";
        case KT_ERR_NULL: return "KT_ERR_NULL: required pointer is NULL";
        case KT_ERR_ALIGN: return "KT_ERR_ALIGN: pointer not aligned for its element type";
        case KT_ERR_LUT: return "KT_ERR_LUT: parameter table would overflow the output mantissa";
        case KT_ERR_SHAPE: return "KT_ERR_SHAPE: unsupported tensor shape";
        case KT_ERR_HIP: return "KT_ERR_HIP: HIP runtime error at launch";
    }
    return "unknown ktanh status";
}

extern "C" const ktanh_lut_t *ktanh_default_lut(void) { return &kTable1; }

// The output mantissa (M >> r) + b must stay a 7-bit unsigned number over the whole interval
// (this is what b_min and b_max of Section 2.4 enforce when a table is fitted); shift-and-add is
// monotone in M, so the interval's first and last mantissa decide.
extern "C" ktanh_status_t ktanh_lut_validate(const ktanh_lut_t *lut)
{
    if (lut == nullptr) return KT_ERR_NULL;
    for (int t = 0; t < KTANH_INTERVALS; ++t) {
        const int E = lut->E[t], r = lut->r[t], b = lut->b[t];
        if (E < 1 || E > 254 || r > 7) return KT_ERR_LUT;
        const int m_first = (t & 7) << 4, m_last = m_first + 15;
        if ((m_first >> r) + b < 0 || (m_last >> r) + b > 127) return KT_ERR_LUT;
    }
    return KT_OK;
}

namespace {

ktanh_status_t pack_slots(const ktanh_lut_t *lut, KtLutPack *pack, bool fold_input_exponent)
{
    if (lut == nullptr) lut = &kTable1;
    const ktanh_status_t st = ktanh_lut_validate(lut);
    if (st != KT_OK) return st;
    // +1.0; the BFloat16 kernels shift the clamped magnitude 0x4080 out entirely, the Float32
    // kernel shifts a zero mantissa
    const uint32_t one = (0x3F80u << 16) | (fold_input_exponent ? 15u : 0u);
    for (int s = 0; s < 64; ++s) pack->slot[s] = one;
    for (int t = 0; t < KTANH_INTERVALS; ++t) {
        // strings 1000..1031 in order of t: 1000 & 31 = 8, and string & 31 = t
        const int string = 1000 + ((t - (1000 & 31)) & 31);
        const int r = lut->r[t];
        int base = (lut->E[t] << 7) + lut->b[t];
        if (fold_input_exponent) base -= (string >> 3) << (7 - r);  // string >> 3 = input exponent
        pack->slot[string & 63] = ((uint32_t)(base & 0xFFFF) << 16) | (uint32_t)r;
    }
    // string 999 (magnitudes 0x3E70..0x3E7F, where the BFloat16 kernels send everything below T1):
    // base 0, shift 0 returns the magnitude itself
    if (fold_input_exponent) pack->slot[999 & 63] = 0u;
    return KT_OK;
}

}  // namespace

ktanh_status_t kt_pack_lut_bf16(const ktanh_lut_t *lut, KtLutPack *pack, bool *within_unit)
{
    if (within_unit != nullptr) {
        const ktanh_lut_t *tab = lut != nullptr ? lut : &kTable1;
        *within_unit = true;
        for (int t = 0; t < KTANH_INTERVALS; ++t) {
            const int last_m = ((t & 7) << 4) + 15;  // shift-and-add is monotone: the last input decides
            const int largest = (tab->E[t] << 7) + (last_m >> (tab->r[t] & 7)) + tab->b[t];
            if (largest > 0x3F80) *within_unit = false;
        }
    }
    return pack_slots(lut, pack, true);
}

ktanh_status_t kt_pack_lut_f32(const ktanh_lut_t *lut, KtLutPack *pack)
{
    return pack_slots(lut, pack, false);
}

// ---- 64-interval variant ------------------------------------------------------------------------
extern "C" ktanh_status_t ktanh_lut64_validate(const ktanh_lut64_t *lut)
{
    if (lut == nullptr) return KT_ERR_NULL;
    for (int t = 0; t < KTANH_INTERVALS64; ++t) {
        const int E = lut->E[t], r = lut->r[t], b = lut->b[t];
        if (E < 1 || E > 254 || r > 7) return KT_ERR_LUT;
        const int m_first = (t & 15) << 3, m_last = m_first + 7;
        if ((m_first >> r) + b < 0 || (m_last >> r) + b > 127) return KT_ERR_LUT;
    }
    return KT_OK;
}

namespace {

const ktanh_lut64_t *fitted_lut64()
{
    static const ktanh_lut64_t fitted = [] {
        ktanh_lut64_t t;
        ktanh_fit_lut64(&t);
        return t;
    }();
    return &fitted;
}

ktanh_status_t pack_slots64(const ktanh_lut64_t *lut, KtLutPack *pack, bool fold_input_exponent)
{
    if (lut == nullptr) lut = fitted_lut64();
    const ktanh_status_t st = ktanh_lut64_validate(lut);
    if (st != KT_OK) return st;
    for (int t = 0; t < KTANH_INTERVALS64; ++t) {
        const int r = lut->r[t];
        // the input exponent in 125..128 whose two low bits are t >> 4
        const int e_in = 125 + ((((t >> 4) & 3) - 125) & 3);
        int base = (lut->E[t] << 7) + lut->b[t];
        if (fold_input_exponent) base -= e_in << (7 - r);
        pack->slot[t] = ((uint32_t)(base & 0xFFFF) << 16) | (uint32_t)r;
    }
    return KT_OK;
}

}  // namespace

ktanh_status_t kt_pack_lut64_bf16(const ktanh_lut64_t *lut, KtLutPack *pack, bool *within_unit)
{
    if (within_unit != nullptr) {
        const ktanh_lut64_t *tab = lut != nullptr ? lut : fitted_lut64();
        *within_unit = true;
        for (int t = 0; t < KTANH_INTERVALS64; ++t) {
            const int last_m = ((t & 15) << 3) + 7;
            const int largest = (tab->E[t] << 7) + (last_m >> (tab->r[t] & 7)) + tab->b[t];
            if (largest > 0x3F80) *within_unit = false;
        }
    }
    return pack_slots64(lut, pack, true);
}

ktanh_status_t kt_pack_lut64_f32(const ktanh_lut64_t *lut, KtLutPack *pack)
{
    return pack_slots64(lut, pack, false);
}

// With y = TanH(a), the derivatives of TanH at a over k! are:  1 - y^2,  -y (1 - y^2),
// -(1 - y^2)(1 - 3 y^2) / 3.
void kt_pack_taylor(KtTaylorPack *pack)
{
    for (int t = 0; t < 32; ++t) {
        const int exponent = ((t >> 3) + 3) % 4 - 2;  // t >> 3 is E & 3 for E = 125..128, i.e. 2^-2..2^1
        const double a = std::ldexp(1.0 + ((t & 7) + 0.5) / 8.0, exponent);
        const double y = std::tanh(a);
        const double slope = 1.0 - y * y;
        pack->c[0][t] = (float)y;
        pack->c[1][t] = (float)slope;
        pack->c[2][t] = (float)(-(y * slope));
        pack->c[3][t] = (float)(-(slope * (1.0 - 3.0 * (y * y))) / 3.0);
    }
}
