// Internal to libktanh: the parameter table in the form the kernels take as an argument.
#pragma once
#include <stdint.h>

#include "ktanh.h"

// One dword per slot of a 64-slot table indexed by the low six bits of the 11-bit string
// (8 exponent bits, 3 leading mantissa bits) that Algorithm 1's threshold tests inspect.
// Strings 1000..1031 (|x| in [0.25, 4)) land on slots 40..63, 0..7 and carry Table 1's entry for
// t = string & 31; string 1032 (|x| clamped to 4) lands on slot 8 and carries the saturation
// value 1.0.  A slot holds  ((E_t << 7) + b_t) << 16  |  r_t : the output magnitude for a zero
// shifted mantissa in the high half, the shift in the low half.
struct KtLutPack {
    uint32_t slot[64];
};

// Validates `lut` (NULL = Table 1) and fills `pack`.
ktanh_status_t kt_pack_lut(const ktanh_lut_t *lut, KtLutPack *pack);
