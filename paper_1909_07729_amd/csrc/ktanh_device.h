// Device-side building blocks of libktanh for gfx950: K-TanH (arXiv:1909.07729, Algorithm 1) on
// packed BFloat16 pairs and on Float32, the derived activations, and the streaming accesses.
//
// The integer work of Algorithm 1 is done on two BFloat16 values per 32-bit register with packed
// 16-bit instructions.  The parameter table is spread over the 64 lanes of each wavefront (one slot
// per lane) and read with ds_bpermute_b32, which needs neither LDS storage nor a barrier.
//
// Because a cross-lane read returns 0 from a disabled lane, every table read executes with the
// whole wavefront enabled: in the kernels, bounds only ever predicate the loads and stores around it.
#pragma once
#include <hip/hip_runtime.h>

#include "ktanh_order.h"
#include "ktanh_pack.h"

namespace ktanh_device {


typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));
typedef int16_t i16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kBlock = 64;  // one wavefront per block: a finished wavefront's slot is refilled at once
// A launch holds fewer than 2^32 work-items: at most this many single-wavefront tiles (64 GiB of
// 128-bit vectors).  Larger tensors are refused before anything is launched.
constexpr unsigned long long kMaxTiles = (1ull << 26) - 1;
constexpr uint32_t kMag2 = 0x7FFF7FFFu;

__device__ __forceinline__ u16x2 as_u16x2(uint32_t w) { return __builtin_bit_cast(u16x2, w); }
__device__ __forceinline__ i16x2 as_i16x2(uint32_t w) { return __builtin_bit_cast(i16x2, w); }
__device__ __forceinline__ uint32_t as_u32(u16x2 v) { return __builtin_bit_cast(uint32_t, v); }
__device__ __forceinline__ uint32_t as_u32(i16x2 v) { return __builtin_bit_cast(uint32_t, v); }
__device__ __forceinline__ u16x2 splat(uint16_t v) { return u16x2{v, v}; }

// 0xFFFF in each 16-bit half whose sign bit is set, 0 elsewhere: one packed arithmetic shift.
// (Written as an instruction because the optimiser would otherwise turn "shift, then select on
// the mask" into per-half compares and selects, which costs three times the issue slots.)
__device__ __forceinline__ uint32_t sign_mask_pair(uint32_t d2)
{
    uint32_t m;
    asm("v_pk_ashrrev_i16 %0, 15, %1 op_sel_hi:[0,1]" : "=v"(m) : "v"(d2));
    return m;
}

// (a & mask) | (b & ~mask): one v_bfi_b32.
__device__ __forceinline__ uint32_t bitsel(uint32_t mask, uint32_t a, uint32_t b)
{
    return (a & mask) | (b & ~mask);
}

// ---------------------------------------------------------------------------------------------
// The parameter table, one slot per lane (KtLutPack layout).  get() takes a byte address whose
// bits [7:2] name the slot; higher bits are ignored by the instruction (lane = address / 4 mod 64).
struct LaneTable {
    uint32_t mine;
    __device__ __forceinline__ explicit LaneTable(const KtLutPack &pack)
        : mine(pack.slot[threadIdx.x & 63])
    {
    }
    __device__ __forceinline__ uint32_t get(uint32_t slot_times_4) const
    {
        return (uint32_t)__builtin_amdgcn_ds_bpermute((int)slot_times_4, (int)mine);
    }
};

// ---------------------------------------------------------------------------------------------
// Algorithm 1 on two BFloat16 magnitudes held in one register (sign bits clear, NaN not handled),
// in two phases so that a caller with several independent pairs can put all their table reads in
// flight before the first result is needed.
//   32 intervals (WIDE = false)
//     slot      = low six bits of (E_i, M_i[6:4]) after clamping |x| to 4.0, so that everything
//                 beyond T2 reads the saturation slot and needs no test of its own;
//     table out = (E_t << 7) + b_t + (M_i >> r_t).  Every slot belongs to one input exponent E_i,
//                 and (|x| >> r) = (E_i << (7 - r)) + (M_i >> r) exactly for r <= 7, so the slot
//                 stores base_t = (E_t << 7) + b_t - (E_i << (7 - r_t)) and the magnitude is
//                 shifted whole: no mantissa mask.  (The saturation slot shifts by 15: 0 is left.)
//     |x| < T1  = one more slot as well: the slot index is taken from max(|x|, 0x3E70), which sends
//                 every magnitude below T1 = 0x3E80 to slot 39 (the index of 0x3E7x), and that slot
//                 holds base 0, shift 0, so the magnitude comes out as it went in.
//   64 intervals (WIDE = true): index = 2 low exponent bits, 4 high mantissa bits; all 64 lanes hold
//     table entries, so saturation is a select of its own.
struct SlotPair {
    uint32_t key2;  // the magnitudes the slots were read for (clamped to 4.0 for 32 intervals)
    uint32_t e_lo, e_hi;
};

template <bool WIDE>
__device__ __forceinline__ SlotPair fetch_slots(uint32_t mag2, const LaneTable &tab)
{
    SlotPair sp;
    if constexpr (WIDE) {
        sp.key2 = mag2;
        sp.e_lo = tab.get(mag2 >> 1);   // bits [7:2] <- bits [8:3] of the low value
        sp.e_hi = tab.get(mag2 >> 17);  // same bits of the high value
    } else {
        sp.key2 = as_u32(__builtin_elementwise_min(as_u16x2(mag2), splat(0x4080)));
        const uint32_t idx2 = as_u32(__builtin_elementwise_max(as_u16x2(sp.key2), splat(0x3E70)));
        sp.e_lo = tab.get(idx2 >> 2);   // bits [7:2] <- bits [9:4] of the low value
        sp.e_hi = tab.get(idx2 >> 18);  // same bits of the high value
    }
    return sp;
}

template <bool WIDE>
__device__ __forceinline__ uint32_t finish_mag_pair(uint32_t mag2, const SlotPair &sp)
{
    const uint32_t base2 = __builtin_amdgcn_perm(sp.e_hi, sp.e_lo, 0x07060302u);
    const uint32_t r2 = __builtin_amdgcn_perm(sp.e_hi, sp.e_lo, 0x05040100u);
    const uint32_t lut2 = as_u32(as_u16x2(base2) + (as_u16x2(sp.key2) >> as_u16x2(r2)));
    if constexpr (!WIDE) return lut2;  // pass-through and saturation are table slots
    // 0xFFFF in each half whose magnitude is below T1 = 0.25 (0x3E80): sign of a 16-bit difference
    const uint32_t pass = sign_mask_pair(as_u32(as_i16x2(mag2) - as_i16x2(0x3E803E80u)));
    const uint32_t res = bitsel(pass, mag2, lut2);
    const uint32_t beyond = sign_mask_pair(as_u32(as_i16x2(0x407F407Fu) - as_i16x2(mag2)));
    return bitsel(beyond, 0x3F803F80u, res);
}

template <bool WIDE = false>
__device__ __forceinline__ uint32_t ktanh_mag_pair(uint32_t mag2, const LaneTable &tab)
{
    return finish_mag_pair<WIDE>(mag2, fetch_slots<WIDE>(mag2, tab));
}

// 0xFFFF in each half that holds a NaN magnitude (> 0x7F80).
__device__ __forceinline__ uint32_t nan_mask_pair(uint32_t mag2)
{
    return sign_mask_pair(as_u32(as_i16x2(0x7F807F80u) - as_i16x2(mag2)));
}

// K-TanH of two BFloat16 values, signs included.  NANS = false leaves out the NaN rule (a NaN then
// comes out as +-1): for callers that have already established that no NaN can reach this point.
template <bool NANS = true, bool WIDE = false>
__device__ __forceinline__ uint32_t ktanh_pair(uint32_t w, const LaneTable &tab)
{
    const uint32_t mag2 = w & kMag2;
    const uint32_t res =
        bitsel(kMag2, ktanh_mag_pair<WIDE>(mag2, tab), w);
    if constexpr (!NANS) return res;
    return bitsel(nan_mask_pair(mag2), w | 0x00400040u, res);
}

// Non-zero where either BFloat16 magnitude of the pair is a NaN (> 0x7F80).
__device__ __forceinline__ uint32_t nan_bits_pair(uint32_t mag2)
{
    return as_u32(__builtin_elementwise_sub_sat(as_u16x2(mag2), splat(0x7F80)));
}
__device__ __forceinline__ uint32_t max_pair(uint32_t a2, uint32_t b2)
{
    return as_u32(__builtin_elementwise_max(as_u16x2(a2), as_u16x2(b2)));
}

// Algorithm 1 on one Float32 pattern: same slot from the same leading bits; the 8-bit parameters
// act on the 23-bit mantissa, b_t aligned to its top seven bits.
template <bool WIDE = false>
__device__ __forceinline__ uint32_t ktanh_f32_one(uint32_t u, const LaneTable &tab)
{
    const uint32_t mag = u & 0x7FFFFFFFu;
    const uint32_t mc = mag < 0x40800000u ? mag : 0x40800000u;
    // 32 intervals: bits [7:2] <- bits [25:20] (slot 8 = saturation); 64 intervals: <- bits [24:19]
    const uint32_t e = tab.get(WIDE ? mag >> 17 : mc >> 18);
    // Float32 slots (kt_pack_lut*_f32) keep the plain base (E_t << 7) + b_t in the high half.
    uint32_t lut = (e & 0xFFFF0000u) + ((mc & 0x007FFFFFu) >> (e & 31u));
    if constexpr (WIDE) lut = mag < 0x40800000u ? lut : 0x3F800000u;
    uint32_t res = mag < 0x3E800000u ? mag : lut;
    res = mag > 0x7F800000u ? (mag | 0x00400000u) : res;
    return res | (u & 0x80000000u);
}

// ---------------------------------------------------------------------------------------------
// BFloat16 <-> Float32.
__device__ __forceinline__ float widen_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float widen_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Two Float32 -> two BFloat16, round to nearest even (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t narrow_pair(float lo, float hi)
{
    const bf16x2 h = __builtin_convertvector(f32x2{lo, hi}, bf16x2);
    return __builtin_bit_cast(uint32_t, h);
}

// Sigmoid: 0.5 * K(0.5 x) + 0.5 in Float32 for both halves of w, in three pieces.
//   Halving a BFloat16 is "exponent field minus one" whenever that field is at least 2; below that
//   |x| < 2^-125, K passes its argument through and the result is 0.5 whatever the argument, so a
//   saturating subtract of 0x80 from the magnitude stands for the multiply and the rounding.
//   0.5 * t is exact for every K output t that can change the sum, so the multiply-add may fuse.
//
// Magnitudes of x/2 for both halves of w (the argument of K inside the Sigmoid).
__device__ __forceinline__ uint32_t sigmoid_half_mag_pair(uint32_t w)
{
    return as_u32(__builtin_elementwise_sub_sat(as_u16x2(w & kMag2), splat(0x0080)));
}

// 0.5 * t + 0.5 for both halves, t = the K output magnitudes `t_mag2` with the signs of w.
template <bool NANS>
__device__ __forceinline__ void sigmoid_from_ktanh_pair(uint32_t w, uint32_t t_mag2, float &s_lo,
                                                        float &s_hi)
{
    uint32_t t2 = bitsel(kMag2, t_mag2, w);
    if constexpr (NANS)
        t2 = bitsel(nan_mask_pair(w & kMag2), w | 0x00400040u, t2);  // NaN in -> NaN through the sums
    s_lo = __builtin_fmaf(0.5f, widen_lo(t2), 0.5f);
    s_hi = __builtin_fmaf(0.5f, widen_hi(t2), 0.5f);
}

template <bool NANS = true, bool WIDE = false>
__device__ __forceinline__ void ksigmoid_f32_pair(uint32_t w, const LaneTable &tab, float &s_lo,
                                                  float &s_hi)
{
    sigmoid_from_ktanh_pair<NANS>(w, ktanh_mag_pair<WIDE>(sigmoid_half_mag_pair(w), tab), s_lo, s_hi);
}

// 128-bit streaming accesses: every byte is touched once.  Measured on tensors that come from HBM:
// loads with the non-temporal hint gain 1-3 % over plain loads (on a tensor its producer left in the
// 256 MB last-level cache the hint costs about 4 %); stores gain about 5 % from the hint and another
// 1-2 % from system-scope write-through (sc0 sc1), which the compiler has no builtin for.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint4 load_stream(const uint4 *p)
{
    const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return uint4{t.x, t.y, t.z, t.w};
}
// The same 16 bytes from an address that is only aligned to its elements (the target allows
// unaligned vector loads; the copy lets the compiler pick a legal access).
__device__ __forceinline__ uint4 load_stream_unaligned(const void *p)
{
    u32x4 t;
    __builtin_memcpy(&t, p, sizeof t);
    return uint4{t.x, t.y, t.z, t.w};
}
// The two idle issue slots after the store belong to it: a store of more than 64 bits reads its
// data registers for a few cycles after issue, and the compiler, which cannot see into the
// statement, may otherwise let the very next instruction overwrite them.
__device__ __forceinline__ void store_stream(uint4 *p, uint4 v)
{
    const u32x4 t = {v.x, v.y, v.z, v.w};
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_nop 1" : : "v"(p), "v"(t) : "memory");
}
// One dword at `base` (uniform) + `byte_offset` (per lane): the hidden outputs of the LSTM cell, a
// thin stream of 256-byte pieces next to four times as many loads.  There the system-scope hint
// alone measured best (2.5-3 % of the kernel over the policy of the 128-bit stores above).
__device__ __forceinline__ void store_stream(uint32_t *base, unsigned byte_offset, uint32_t v)
{
    asm volatile("global_store_dword %0, %1, %2 sc1"
                 :
                 : "v"(byte_offset), "v"(v), "s"(base)
                 : "memory");
}

// OP_COPY moves the data unchanged: the same accesses with no arithmetic, the yardstick for what the
// memory system allows in this launch shape.
// OP_PADE32 / OP_PADE78: the rational approximants of Section 2 that Table 2 compares K-TanH with.
// OP_TAYLOR2 / OP_TAYLOR3: piecewise Taylor polynomials on K-TanH's own intervals, for Table 2's Taylor rows.
enum Op {
    OP_TANH = 0, OP_SIGMOID = 1, OP_SWISH = 2, OP_GELU = 3, OP_COPY = 4, OP_PADE32 = 5, OP_PADE78 = 6,
    OP_TAYLOR2 = 7, OP_TAYLOR3 = 8
};

// Pade[3/2] = x (15 + x^2) / (15 + 6 x^2) on min(|x|, 4), capped at 1;
// Pade[7/8] = x (2027025 + 270270 x^2 + 6930 x^4 + 36 x^6) / (2027025 + 945945 x^2 + 51975 x^4 + 630 x^6 + x^8)
// on min(|x|, 5.5).  Float32, one rounding per operation (Horner in x^2), correctly rounded division.
template <int OP>
__device__ __forceinline__ float pade_of_magnitude(float a)
{
    if constexpr (OP == OP_PADE32) {
        a = a > 4.0f ? 4.0f : a;
        const float x2 = a * a;
        const float num = a * (15.0f + x2);
        const float den = 15.0f + 6.0f * x2;
        const float y = num / den;
        return y > 1.0f ? 1.0f : y;
    } else {
        a = a > 5.5f ? 5.5f : a;
        const float x2 = a * a;
        float p = 36.0f * x2 + 6930.0f;
        p = p * x2 + 270270.0f;
        p = p * x2 + 2027025.0f;
        const float num = a * p;
        float q = x2 + 630.0f;
        q = q * x2 + 51975.0f;
        q = q * x2 + 945945.0f;
        q = q * x2 + 2027025.0f;
        return num / q;
    }
}

// Both halves of w: magnitudes through the approximant, signs put back, NaNs returned quieted.
template <int OP>
__device__ __forceinline__ uint32_t pade_pair(uint32_t w)
{
    const uint32_t mag2 = w & kMag2;
    const uint32_t y2 = narrow_pair(pade_of_magnitude<OP>(widen_lo(mag2)), pade_of_magnitude<OP>(widen_hi(mag2)));
    const uint32_t res = bitsel(kMag2, y2, w);
    return bitsel(nan_mask_pair(mag2), w | 0x00400040u, res);
}

// The coefficient table of the Taylor polynomials, spread over the lanes like the K-TanH table: lane
// l holds the four coefficients of interval l & 31 (both halves of the wavefront hold all 32).
struct TaylorLane {
    float c[4];
    __device__ __forceinline__ explicit TaylorLane(const KtTaylorPack &pack)
    {
        const unsigned t = threadIdx.x & 31;
#pragma unroll
        for (int k = 0; k < 4; ++k) c[k] = pack.c[k][t];
    }
    // Coefficient k of the interval named by bits [6:2] of the byte address (bit 7 picks one of the
    // two lanes that hold it, higher bits are ignored).  Every lane of the wavefront must be enabled.
    __device__ __forceinline__ float get(int k, uint32_t t_times_4) const
    {
        return __uint_as_float(
            (uint32_t)__builtin_amdgcn_ds_bpermute((int)t_times_4, (int)__float_as_uint(c[k])));
    }
};

// T_n(|x|) = sum_k c_k (|x| - a_t)^k for one BFloat16 magnitude in [0.25, 4) (bits 0..15 of `mag`);
// anything for magnitudes outside.  Float32, Horner's scheme, one rounding per operation.  The
// interval's midpoint a_t is the magnitude with its four low mantissa bits replaced by 1000, and
// the difference is exact.
template <int DEGREE>
__device__ __forceinline__ float taylor_of_magnitude(uint32_t mag, const TaylorLane &tab)
{
    const uint32_t at = mag >> 2;  // bits [6:2] <- bits [8:4] of the magnitude: t
    const float h = __uint_as_float(mag << 16) - __uint_as_float(((mag & 0x7FF0u) | 0x0008u) << 16);
    float p = tab.get(DEGREE, at);
#pragma unroll
    for (int k = DEGREE - 1; k >= 0; --k) {
        p = p * h;
        p = p + tab.get(k, at);
    }
    return p;
}

// Both halves of w: the regions of Algorithm 1 (pass-through below 0.25, 1 from 4.0 on), the
// polynomial in between, signs put back, NaNs returned quieted.
template <int OP>
__device__ __forceinline__ uint32_t taylor_pair(uint32_t w, const TaylorLane &tab)
{
    constexpr int DEGREE = OP == OP_TAYLOR3 ? 3 : 2;
    const uint32_t mag2 = w & kMag2;
    const uint32_t y2 = narrow_pair(taylor_of_magnitude<DEGREE>(mag2 & 0xFFFFu, tab),
                                    taylor_of_magnitude<DEGREE>(mag2 >> 16, tab));
    const uint32_t pass = sign_mask_pair(as_u32(as_i16x2(mag2) - as_i16x2(0x3E803E80u)));
    const uint32_t beyond = sign_mask_pair(as_u32(as_i16x2(0x407F407Fu) - as_i16x2(mag2)));
    uint32_t res = bitsel(pass, mag2, y2);
    res = bitsel(beyond, 0x3F803F80u, res);
    res = bitsel(kMag2, res, w);
    return bitsel(nan_mask_pair(mag2), w | 0x00400040u, res);
}

// The kernel-argument form and the per-lane form of the table an operation reads.
template <int OP>
struct TableOf {
    typedef KtLutPack Pack;
    typedef LaneTable Lane;
};
template <>
struct TableOf<OP_TAYLOR2> {
    typedef KtTaylorPack Pack;
    typedef TaylorLane Lane;
};
template <>
struct TableOf<OP_TAYLOR3> {
    typedef KtTaylorPack Pack;
    typedef TaylorLane Lane;
};

// WIDE selects the 64-interval table layout.
template <int OP, bool WIDE = false, class Tab>
__device__ __forceinline__ uint32_t apply_pair(uint32_t w, const Tab &tab)
{
    if constexpr (OP == OP_COPY) {
        return w;
    } else if constexpr (OP == OP_PADE32 || OP == OP_PADE78) {
        return pade_pair<OP>(w);
    } else if constexpr (OP == OP_TAYLOR2 || OP == OP_TAYLOR3) {
        return taylor_pair<OP>(w, tab);
    } else if constexpr (OP == OP_TANH) {
        return ktanh_pair<true, WIDE>(w, tab);
    } else if constexpr (OP == OP_SIGMOID) {
        float s_lo, s_hi;
        ksigmoid_f32_pair<true, WIDE>(w, tab, s_lo, s_hi);
        return narrow_pair(s_lo, s_hi);
    } else if constexpr (OP == OP_SWISH) {
        // No NaN rule inside: the product with x makes a NaN input a NaN output whatever K returns.
        float s_lo, s_hi;
        ksigmoid_f32_pair<false, WIDE>(w, tab, s_lo, s_hi);
        return narrow_pair(widen_lo(w) * s_lo, widen_hi(w) * s_hi);
    } else {
        // GELU, tanh form: (x/2) * (1 + K(c * (x + a * x^3))).  (x/2) * (1 + t) and
        // x * (0.5 + 0.5 t) are the same real product and round alike (halving is exact).
        const float a = 0.044715f;
        const float c = 0.7978845608028654f;
        const float x_lo = widen_lo(w), x_hi = widen_hi(w);
        const float u_lo = c * (x_lo + a * ((x_lo * x_lo) * x_lo));
        const float u_hi = c * (x_hi + a * ((x_hi * x_hi) * x_hi));
        // The argument is a NaN only where x is one (x + a x^3 cannot cancel: both terms carry the
        // sign of x), and there the last product is a NaN whatever K returns: no NaN rule inside.
        const uint32_t t2 = ktanh_pair<false, WIDE>(narrow_pair(u_lo, u_hi), tab);
        const float y_lo = x_lo * __builtin_fmaf(0.5f, widen_lo(t2), 0.5f);
        const float y_hi = x_hi * __builtin_fmaf(0.5f, widen_hi(t2), 0.5f);
        return narrow_pair(y_lo, y_hi);
    }
}

template <int OP, bool WIDE = false, class Tab>
__device__ __forceinline__ uint4 apply_vec_bf16(uint4 v, const Tab &tab)
{
    return uint4{apply_pair<OP, WIDE>(v.x, tab), apply_pair<OP, WIDE>(v.y, tab),
                 apply_pair<OP, WIDE>(v.z, tab), apply_pair<OP, WIDE>(v.w, tab)};
}

// One Float32 element of a Float32-tensor operation.
//   Sigmoid: 0.5 * t is exact for every K output t that can change the sum, so multiply-add fuses.
//   GELU: (x/2) * (1 + t) and x * (0.5 + 0.5 t) are the same real product and round alike.
template <int OP, bool WIDE = false>
__device__ __forceinline__ uint32_t apply_f32_one(uint32_t u, const LaneTable &tab)
{
    if constexpr (OP == OP_TANH) {
        return ktanh_f32_one<WIDE>(u, tab);
    } else if constexpr (OP == OP_SIGMOID || OP == OP_SWISH) {
        const float x = __uint_as_float(u);
        const float t = __uint_as_float(ktanh_f32_one<WIDE>(__float_as_uint(0.5f * x), tab));
        const float sg = __builtin_fmaf(0.5f, t, 0.5f);
        return __float_as_uint(OP == OP_SIGMOID ? sg : x * sg);
    } else {
        const float a = 0.044715f;
        const float c = 0.7978845608028654f;
        const float x = __uint_as_float(u);
        const float arg = c * (x + a * ((x * x) * x));
        const float t = __uint_as_float(ktanh_f32_one<WIDE>(__float_as_uint(arg), tab));
        return __float_as_uint(x * __builtin_fmaf(0.5f, t, 0.5f));
    }
}

template <int OP, bool WIDE = false>
__device__ __forceinline__ uint4 apply_vec_f32(uint4 v, const LaneTable &tab)
{
    return uint4{apply_f32_one<OP, WIDE>(v.x, tab), apply_f32_one<OP, WIDE>(v.y, tab),
                 apply_f32_one<OP, WIDE>(v.z, tab), apply_f32_one<OP, WIDE>(v.w, tab)};
}

// Which table layout a caller's table type selects.
constexpr bool is_wide(const ktanh_lut_t *) { return false; }
constexpr bool is_wide(const ktanh_lut64_t *) { return true; }

// Enqueues `kernel` and returns the status of this very launch (the launch macro would only leave it
// in the runtime's last-error slot, next to whatever an earlier, unrelated call left there).
template <class... Params, class... Args>
inline ktanh_status_t launch_checked(void (*kernel)(Params...), unsigned blocks, unsigned threads,
                                     ktanh_stream_t stream, Args... args)
{
    static_assert(sizeof...(Params) == sizeof...(Args), "argument count");
    // each argument converted to the kernel's parameter type, then passed by address
    auto call = [&](Params... converted) {
        void *slots[] = {static_cast<void *>(&converted)...};
        return hipLaunchKernel(reinterpret_cast<const void *>(kernel), dim3(blocks), dim3(threads),
                               slots, 0, static_cast<hipStream_t>(stream));
    };
    return call(args...) == hipSuccess ? KT_OK : KT_ERR_HIP;
}

}  // namespace ktanh_device
