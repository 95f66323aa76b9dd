// Internal to libktanh: the parameter table in the form the kernels take as an argument.
#pragma once
#include <stdint.h>

#include "ktanh.h"

// One dword per slot of a 64-slot table indexed by the low six bits of the 11-bit string
// (8 exponent bits, 3 leading mantissa bits) that Algorithm 1's threshold tests inspect.
// Strings 1000..1031 (|x| in [0.25, 4)) land on slots 40..63, 0..7 and carry Table 1's entry for
// t = string & 31; string 1032 (|x| clamped to 4) lands on slot 8 and carries the saturation
// value 1.0.  A slot holds  base << 16 | shift :
//   BFloat16 kernels: base = (E_t << 7) + b_t - (E_i << (7 - r_t)), E_i the input exponent the slot
//                     belongs to, so that base + (|x| >> r_t) is the output magnitude with no
//                     mantissa mask; shift = r_t (15 in the saturation slot: |x| >> 15 = 0);
//   Float32 kernel:   base = (E_t << 7) + b_t, to be aligned to the top of the word and added to
//                     the shifted 23-bit mantissa; shift = r_t.
struct KtLutPack {
    uint32_t slot[64];
};

// Validate `lut` (NULL = Table 1) and fill `pack` for the BFloat16 kernels / the Float32 kernel.
// `within_unit` (optional) is set to whether no table output can exceed 1.0 in magnitude, as is the
// case for any table fitted to TanH; a caller's table may break it.
ktanh_status_t kt_pack_lut_bf16(const ktanh_lut_t *lut, KtLutPack *pack, bool *within_unit = nullptr);
ktanh_status_t kt_pack_lut_f32(const ktanh_lut_t *lut, KtLutPack *pack);

// 64-interval tables: slot = t = (E_i & 3) << 4 | (M_i >> 3), all 64 slots are table entries (the
// saturation value has no slot of its own; the kernels select it).  Same slot format as above.
// NULL = the fitted 64-interval table.
ktanh_status_t kt_pack_lut64_bf16(const ktanh_lut64_t *lut, KtLutPack *pack,
                                  bool *within_unit = nullptr);
ktanh_status_t kt_pack_lut64_f32(const ktanh_lut64_t *lut, KtLutPack *pack);

// The piecewise Taylor polynomials of TanH that stand in for Table 2's two Taylor rows: for each of
// Table 1's 32 intervals (index t = 2 low exponent bits, 3 high mantissa bits of |x| in [0.25, 4))
// the coefficients of (|x| - a_t)^k, k = 0..3, about the interval's midpoint a_t, formed in double
// precision and rounded to Float32.  c[k][t].
struct KtTaylorPack {
    float c[4][32];
};
void kt_pack_taylor(KtTaylorPack *pack);
