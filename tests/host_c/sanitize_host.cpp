// Host-only sources of the library (table, validation, packing, fit) under AddressSanitizer and
// UndefinedBehaviorSanitizer: built and run by tests/test_boundary_host.py with g++, no GPU involved.
#include <cstdio>
#include <cstring>

#include "ktanh_pack.h"

int main()
{
    ktanh_lut_t fitted;
    ktanh_lut64_t fitted64;
    if (ktanh_fit_lut(&fitted) != KT_OK) return 1;
    if (std::memcmp(&fitted, ktanh_default_lut(), sizeof fitted) != 0) return 2;
    if (ktanh_fit_lut64(&fitted64) != KT_OK || ktanh_lut64_validate(&fitted64) != KT_OK) return 3;
    KtLutPack pack;
    if (kt_pack_lut_bf16(nullptr, &pack) != KT_OK || kt_pack_lut_f32(&fitted, &pack) != KT_OK) return 4;
    if (kt_pack_lut64_bf16(nullptr, &pack) != KT_OK || kt_pack_lut64_f32(&fitted64, &pack) != KT_OK) return 5;
    // every extreme a validated table may hold
    for (int t = 0; t < KTANH_INTERVALS; ++t) { fitted.E[t] = 254; fitted.r[t] = 7; fitted.b[t] = 127; }
    if (ktanh_lut_validate(&fitted) != KT_OK || kt_pack_lut_bf16(&fitted, &pack) != KT_OK) return 6;
    for (int t = 0; t < KTANH_INTERVALS; ++t) { fitted.E[t] = 1; fitted.r[t] = 0; fitted.b[t] = (int8_t)(-((t & 7) << 4)); }
    if (ktanh_lut_validate(&fitted) != KT_OK || kt_pack_lut_bf16(&fitted, &pack) != KT_OK) return 7;
    fitted.b[5] = -128;
    if (ktanh_lut_validate(&fitted) != KT_ERR_LUT) return 8;
    std::puts("host sources clean");
    return 0;
}
