// libktanh device code and entry points: K-TanH (arXiv:1909.07729, Algorithm 1) and the
// activations built on it, for gfx950.
//
// Shape of every kernel: a pure HBM stream.  Each lane moves 128 bits per access (8 BFloat16 or
// 4 Float32), a wavefront covers 1 KiB per access, several accesses are in flight per lane, and the
// integer work of Algorithm 1 is done on two BFloat16 values per 32-bit register with packed 16-bit
// instructions.  The parameter table is spread over the 64 lanes of each wavefront (one slot per
// lane) and read with ds_bpermute_b32, which needs neither LDS storage nor a barrier.
//
// Because a cross-lane read returns 0 from a disabled lane, every table read below executes with
// the whole wavefront enabled: bounds only ever predicate the loads and stores around it.
#include <hip/hip_runtime.h>

#include "ktanh_pack.h"

namespace {

typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));
typedef int16_t i16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kBlock = 256;   // 4 wavefronts
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
// Algorithm 1 on two BFloat16 magnitudes held in one register (sign bits clear, NaN not handled).
//   slot      = low six bits of (E_i, M_i[6:4]) after clamping |x| to 4.0, so that everything
//               beyond T2 reads the saturation slot and needs no test of its own;
//   table out = (E_t << 7) + b_t + (M_i >> r_t).  Every slot belongs to one input exponent E_i, and
//               (|x| >> r) = (E_i << (7 - r)) + (M_i >> r) exactly for r <= 7, so the slot stores
//               base_t = (E_t << 7) + b_t - (E_i << (7 - r_t)) and the magnitude is shifted whole:
//               no mantissa mask.  (The saturation slot shifts by 15, which leaves 0.)
//   |x| < T1  = input passed through.
__device__ __forceinline__ uint32_t ktanh_mag_pair(uint32_t mag2, const LaneTable &tab)
{
    const uint32_t mc2 = as_u32(__builtin_elementwise_min(as_u16x2(mag2), splat(0x4080)));
    const uint32_t e_lo = tab.get(mc2 >> 2);   // bits [7:2] <- bits [9:4] of the low value
    const uint32_t e_hi = tab.get(mc2 >> 18);  // same bits of the high value
    const uint32_t base2 = __builtin_amdgcn_perm(e_hi, e_lo, 0x07060302u);
    const uint32_t r2 = __builtin_amdgcn_perm(e_hi, e_lo, 0x05040100u);
    const uint32_t lut2 = as_u32(as_u16x2(base2) + (as_u16x2(mc2) >> as_u16x2(r2)));
    // 0xFFFF in each half whose magnitude is below T1 = 0.25 (0x3E80): sign of a 16-bit difference
    const uint32_t pass = sign_mask_pair(as_u32(as_i16x2(mag2) - as_i16x2(0x3E803E80u)));
    return bitsel(pass, mag2, lut2);
}

// The same with a 64-interval table (index = 2 low exponent bits, 4 high mantissa bits): all 64
// lanes hold table entries, so saturation is a select of its own.
__device__ __forceinline__ uint32_t ktanh64_mag_pair(uint32_t mag2, const LaneTable &tab)
{
    const uint32_t e_lo = tab.get(mag2 >> 1);   // bits [7:2] <- bits [8:3] of the low value
    const uint32_t e_hi = tab.get(mag2 >> 17);  // same bits of the high value
    const uint32_t base2 = __builtin_amdgcn_perm(e_hi, e_lo, 0x07060302u);
    const uint32_t r2 = __builtin_amdgcn_perm(e_hi, e_lo, 0x05040100u);
    const uint32_t lut2 = as_u32(as_u16x2(base2) + (as_u16x2(mag2) >> as_u16x2(r2)));
    const uint32_t pass = sign_mask_pair(as_u32(as_i16x2(mag2) - as_i16x2(0x3E803E80u)));
    const uint32_t beyond = sign_mask_pair(as_u32(as_i16x2(0x407F407Fu) - as_i16x2(mag2)));
    return bitsel(beyond, 0x3F803F80u, bitsel(pass, mag2, lut2));
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
        bitsel(kMag2, WIDE ? ktanh64_mag_pair(mag2, tab) : ktanh_mag_pair(mag2, tab), w);
    if constexpr (!NANS) return res;
    return bitsel(nan_mask_pair(mag2), w | 0x00400040u, res);
}

// True in a lane where any of the given BFloat16 magnitude pairs holds a NaN.
__device__ __forceinline__ bool any_nan_pair(uint32_t mag2)
{
    return as_u32(__builtin_elementwise_sub_sat(as_u16x2(mag2), splat(0x7F80))) != 0u;
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

// 0.5 * K(0.5 x) + 0.5 in Float32 for both halves of w.
//   Halving a BFloat16 is "exponent field minus one" whenever that field is at least 2; below that
//   |x| < 2^-125, K passes its argument through and the result is 0.5 whatever the argument, so a
//   saturating subtract of 0x80 from the magnitude stands for the multiply and the rounding.
//   0.5 * t is exact for every K output t that can change the sum, so the multiply-add may fuse.
template <bool NANS = true>
__device__ __forceinline__ void ksigmoid_f32_pair(uint32_t w, const LaneTable &tab, float &s_lo,
                                                  float &s_hi)
{
    const uint32_t mag2 = w & kMag2;
    const uint32_t half_mag2 = as_u32(__builtin_elementwise_sub_sat(as_u16x2(mag2), splat(0x0080)));
    uint32_t t2 = bitsel(kMag2, ktanh_mag_pair(half_mag2, tab), w);
    if constexpr (NANS)
        t2 = bitsel(nan_mask_pair(mag2), w | 0x00400040u, t2);  // NaN in -> NaN through the sums
    s_lo = __builtin_fmaf(0.5f, widen_lo(t2), 0.5f);
    s_hi = __builtin_fmaf(0.5f, widen_hi(t2), 0.5f);
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
__device__ __forceinline__ void store_stream(uint4 *p, uint4 v)
{
    const u32x4 t = {v.x, v.y, v.z, v.w};
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt" : : "v"(p), "v"(t) : "memory");
}
// One dword at `base` (uniform) + `byte_offset` (per lane).
__device__ __forceinline__ void store_stream(uint32_t *base, unsigned byte_offset, uint32_t v)
{
    asm volatile("global_store_dword %0, %1, %2 sc0 sc1 nt"
                 :
                 : "v"(byte_offset), "v"(v), "s"(base)
                 : "memory");
}

enum Op { OP_TANH = 0, OP_SIGMOID = 1, OP_SWISH = 2, OP_GELU = 3, OP_TANH64 = 4 };

template <int OP>
__device__ __forceinline__ uint32_t apply_pair(uint32_t w, const LaneTable &tab)
{
    if constexpr (OP == OP_TANH) {
        return ktanh_pair(w, tab);
    } else if constexpr (OP == OP_TANH64) {
        return ktanh_pair<true, true>(w, tab);
    } else if constexpr (OP == OP_SIGMOID) {
        float s_lo, s_hi;
        ksigmoid_f32_pair(w, tab, s_lo, s_hi);
        return narrow_pair(s_lo, s_hi);
    } else if constexpr (OP == OP_SWISH) {
        float s_lo, s_hi;
        ksigmoid_f32_pair(w, tab, s_lo, s_hi);
        return narrow_pair(widen_lo(w) * s_lo, widen_hi(w) * s_hi);
    } else {
        // GELU, tanh form: (x/2) * (1 + K(c * (x + a * x^3))).  (x/2) * (1 + t) and
        // x * (0.5 + 0.5 t) are the same real product and round alike (halving is exact).
        const float a = 0.044715f;
        const float c = 0.7978845608028654f;
        const float x_lo = widen_lo(w), x_hi = widen_hi(w);
        const float u_lo = c * (x_lo + a * ((x_lo * x_lo) * x_lo));
        const float u_hi = c * (x_hi + a * ((x_hi * x_hi) * x_hi));
        const uint32_t t2 = ktanh_pair(narrow_pair(u_lo, u_hi), tab);
        const float y_lo = x_lo * __builtin_fmaf(0.5f, widen_lo(t2), 0.5f);
        const float y_hi = x_hi * __builtin_fmaf(0.5f, widen_hi(t2), 0.5f);
        return narrow_pair(y_lo, y_hi);
    }
}

template <int OP>
__device__ __forceinline__ uint4 apply_vec_bf16(uint4 v, const LaneTable &tab)
{
    return uint4{apply_pair<OP>(v.x, tab), apply_pair<OP>(v.y, tab), apply_pair<OP>(v.z, tab),
                 apply_pair<OP>(v.w, tab)};
}

// One Float32 element of a Float32-tensor operation.
//   Sigmoid: 0.5 * t is exact for every K output t that can change the sum, so multiply-add fuses.
//   GELU: (x/2) * (1 + t) and x * (0.5 + 0.5 t) are the same real product and round alike.
template <int OP>
__device__ __forceinline__ uint32_t apply_f32_one(uint32_t u, const LaneTable &tab)
{
    if constexpr (OP == OP_TANH || OP == OP_TANH64) {
        return ktanh_f32_one<OP == OP_TANH64>(u, tab);
    } else if constexpr (OP == OP_SIGMOID || OP == OP_SWISH) {
        const float x = __uint_as_float(u);
        const float t = __uint_as_float(ktanh_f32_one(__float_as_uint(0.5f * x), tab));
        const float sg = __builtin_fmaf(0.5f, t, 0.5f);
        return __float_as_uint(OP == OP_SIGMOID ? sg : x * sg);
    } else {
        const float a = 0.044715f;
        const float c = 0.7978845608028654f;
        const float x = __uint_as_float(u);
        const float arg = c * (x + a * ((x * x) * x));
        const float t = __uint_as_float(ktanh_f32_one(__float_as_uint(arg), tab));
        return __float_as_uint(x * __builtin_fmaf(0.5f, t, 0.5f));
    }
}

template <int OP>
__device__ __forceinline__ uint4 apply_vec_f32(uint4 v, const LaneTable &tab)
{
    return uint4{apply_f32_one<OP>(v.x, tab), apply_f32_one<OP>(v.y, tab),
                 apply_f32_one<OP>(v.z, tab), apply_f32_one<OP>(v.w, tab)};
}

// ---------------------------------------------------------------------------------------------
// Element-wise streaming kernel over `nvec` 128-bit vectors plus up to `n_edge` loose elements.
//   vin, vout : 16-byte aligned body (nvec vectors)
//   ein, eout : the whole tensor as elements; edge element k (k < n_head) is element k, edge
//               element k >= n_head is element n_total - n_edge + k (the ragged tail)
// F32 selects the Float32 K-TanH (OP ignored), else the BFloat16 operation OP.
struct EdgeArgs {
    const void *ein;
    void *eout;
    unsigned long long n_total;
    unsigned n_head;
    unsigned n_edge;  // head + tail elements, < 64
};

template <bool F32, int OP>
__device__ __forceinline__ uint4 apply_vec(uint4 v, const LaneTable &tab)
{
    if constexpr (F32) return apply_vec_f32<OP>(v, tab);
    else return apply_vec_bf16<OP>(v, tab);
}

template <bool F32, int OP, int kUnroll>
__global__ __launch_bounds__(kBlock) void stream_kernel(const uint4 *__restrict__ vin,
                                                        uint4 *__restrict__ vout,
                                                        unsigned long long nvec, EdgeArgs edge,
                                                        KtLutPack pack)
{
    const LaneTable tab(pack);

    // One tile of kBlock * kUnroll vectors per block, no loop: fresh blocks keep loads and stores
    // of different tiles overlapped, which a grid-stride loop over the same tiles does not (measured:
    // 6.5 against 6.0 TB/s on a 537 MB stream).  kUnroll = 1 moves the most bytes for the light
    // operations; the Float32-heavy ones need two vectors per lane to hide their arithmetic.
    const unsigned long long at = (unsigned long long)blockIdx.x * (kBlock * kUnroll) + threadIdx.x;
    uint4 v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        v[u] = uint4{0u, 0u, 0u, 0u};
        if (at + (unsigned long long)u * kBlock < nvec) v[u] = load_stream(vin + at + u * kBlock);
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) v[u] = apply_vec<F32, OP>(v[u], tab);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
        if (at + (unsigned long long)u * kBlock < nvec) store_stream(vout + at + u * kBlock, v[u]);

    // Loose elements before and after the aligned body: first wavefront of block 0.
    if (edge.n_edge != 0 && blockIdx.x == 0 && threadIdx.x < 64) {
        const unsigned k = threadIdx.x;
        const bool live = k < edge.n_edge;
        const unsigned long long i =
            k < edge.n_head ? k : edge.n_total - edge.n_edge + k;
        uint32_t x = 0;
        if constexpr (F32) {
            if (live) x = static_cast<const uint32_t *>(edge.ein)[i];
            x = apply_f32_one<OP>(x, tab);
            if (live) static_cast<uint32_t *>(edge.eout)[i] = x;
        } else {
            if (live) x = static_cast<const uint16_t *>(edge.ein)[i];
            x = apply_pair<OP>(x, tab);
            if (live) static_cast<uint16_t *>(edge.eout)[i] = (uint16_t)x;
        }
    }
}

// Fallback when `in` and `out` disagree modulo 16 bytes: one element per lane and pass.
template <bool F32, int OP>
__global__ __launch_bounds__(kBlock) void element_kernel(const void *__restrict__ in,
                                                         void *__restrict__ out,
                                                         unsigned long long n, KtLutPack pack)
{
    const LaneTable tab(pack);
    const unsigned long long stride = (unsigned long long)gridDim.x * kBlock;
    for (unsigned long long base = (unsigned long long)blockIdx.x * kBlock; base < n;
         base += stride) {
        const unsigned long long i = base + threadIdx.x;
        const bool live = i < n;
        uint32_t x = 0;
        if constexpr (F32) {
            if (live) x = static_cast<const uint32_t *>(in)[i];
            x = apply_f32_one<OP>(x, tab);
            if (live) static_cast<uint32_t *>(out)[i] = x;
        } else {
            if (live) x = static_cast<const uint16_t *>(in)[i];
            x = apply_pair<OP>(x, tab);
            if (live) static_cast<uint16_t *>(out)[i] = (uint16_t)x;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Float32 in, BFloat16 out: round to nearest even (v_cvt_pk_bf16_f32), then K-TanH.  Each lane
// reads two 128-bit vectors (4 Float32 each) and writes two 64-bit ones.
__device__ __forceinline__ void store_stream(uint2 *p, uint2 v)
{
    asm volatile("global_store_dwordx2 %0, %1, off sc0 sc1 nt" : : "v"(p), "v"(v) : "memory");
}

__device__ __forceinline__ uint2 narrow_ktanh_vec(uint4 v, const LaneTable &tab)
{
    const uint32_t w0 = narrow_pair(__uint_as_float(v.x), __uint_as_float(v.y));
    const uint32_t w1 = narrow_pair(__uint_as_float(v.z), __uint_as_float(v.w));
    return uint2{ktanh_pair(w0, tab), ktanh_pair(w1, tab)};
}

__global__ __launch_bounds__(kBlock) void narrow_stream_kernel(const uint4 *__restrict__ vin,
                                                               uint2 *__restrict__ vout,
                                                               unsigned long long nvec,
                                                               EdgeArgs edge, KtLutPack pack)
{
    const LaneTable tab(pack);
    const unsigned long long at = (unsigned long long)blockIdx.x * (kBlock * 2) + threadIdx.x;
    uint4 v[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        v[u] = uint4{0u, 0u, 0u, 0u};
        if (at + (unsigned long long)u * kBlock < nvec) v[u] = load_stream(vin + at + u * kBlock);
    }
    uint2 o[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) o[u] = narrow_ktanh_vec(v[u], tab);
#pragma unroll
    for (int u = 0; u < 2; ++u)
        if (at + (unsigned long long)u * kBlock < nvec) store_stream(vout + at + u * kBlock, o[u]);

    if (edge.n_edge != 0 && blockIdx.x == 0 && threadIdx.x < 64) {
        const unsigned k = threadIdx.x;
        const bool live = k < edge.n_edge;
        const unsigned long long i = k < edge.n_head ? k : edge.n_total - edge.n_edge + k;
        uint32_t x = 0;
        if (live) x = static_cast<const uint32_t *>(edge.ein)[i];
        x = ktanh_pair(narrow_pair(__uint_as_float(x), 0.0f), tab);
        if (live) static_cast<uint16_t *>(edge.eout)[i] = (uint16_t)x;
    }
}

__global__ __launch_bounds__(kBlock) void narrow_element_kernel(const uint32_t *__restrict__ in,
                                                                uint16_t *__restrict__ out,
                                                                unsigned long long n, KtLutPack pack)
{
    const LaneTable tab(pack);
    const unsigned long long stride = (unsigned long long)gridDim.x * kBlock;
    for (unsigned long long base = (unsigned long long)blockIdx.x * kBlock; base < n;
         base += stride) {
        const unsigned long long i = base + threadIdx.x;
        const bool live = i < n;
        uint32_t x = 0;
        if (live) x = in[i];
        x = ktanh_pair(narrow_pair(__uint_as_float(x), 0.0f), tab);
        if (live) out[i] = (uint16_t)x;
    }
}

// ---------------------------------------------------------------------------------------------
// LSTM cell: each lane owns two neighbouring cells of one batch row (one packed BFloat16 pair per
// gate) and carries their state through all T steps.  The work per cell is about sixty vector
// instructions against ten bytes of traffic, so the kernel wants many wavefronts per SIMD to overlap
// arithmetic with memory rather than wide accesses; a wavefront's loads still cover 256 contiguous
// bytes each.  The steps of one lane are sequential, so the gate words of the next kStages steps are
// already on their way while a step is computed (a ring of register stages): without that the loop
// would pay one full memory latency per step.
constexpr int kStages = 4;

struct GateWords {
    uint32_t i, f, g, o;
};

// Byte offsets of a lane's four gate words inside one time step's [B][4H] gate matrix: 32-bit, so
// that each load is "uniform 64-bit base + 32-bit lane offset" and needs no address arithmetic.
struct GateOffsets {
    unsigned i, f, g, o;
};

__device__ __forceinline__ uint32_t load_word(const uint32_t *base, unsigned byte_offset)
{
    return *reinterpret_cast<const uint32_t *>(reinterpret_cast<const char *>(base) + byte_offset);
}

__device__ __forceinline__ GateWords load_gates(const uint32_t *step_base, GateOffsets &at,
                                                bool live)
{
    // The empty statement re-defines the four 32-bit offsets right where they are used, so that
    // each access is selected as "scalar base + 32-bit vector offset"; otherwise their 64-bit
    // extensions are hoisted out of the loop and every access pays a 64-bit vector add.
    asm volatile("" : "+v"(at.i), "+v"(at.f), "+v"(at.g), "+v"(at.o));
    GateWords q{0u, 0u, 0u, 0u};
    if (live) {
        q.i = load_word(step_base, at.i);
        q.f = load_word(step_base, at.f);
        q.g = load_word(step_base, at.g);
        q.o = load_word(step_base, at.o);
    }
    return q;
}

__device__ __forceinline__ bool not_finite(float x)
{
    return (__float_as_uint(x) & 0x7F800000u) == 0x7F800000u;
}

// One time step for the two cells of a lane: updates their state, returns the two hidden outputs.
// NANS = false is the same arithmetic without the NaN rules of K-TanH; it is exact whenever no gate
// is NaN and the incoming state is finite (the state then stays finite: |c'| <= |c| + 1).
template <bool NANS>
__device__ __forceinline__ uint32_t lstm_step(const GateWords &q, float &c_lo, float &c_hi,
                                              const LaneTable &tab)
{
    float i_lo, i_hi, f_lo, f_hi, o_lo, o_hi;
    ksigmoid_f32_pair<NANS>(q.i, tab, i_lo, i_hi);
    ksigmoid_f32_pair<NANS>(q.f, tab, f_lo, f_hi);
    ksigmoid_f32_pair<NANS>(q.o, tab, o_lo, o_hi);
    const uint32_t g2 = ktanh_pair<NANS>(q.g, tab);
    // c' = (f * c) + (i * g): two products and one sum, each rounded on its own
    const float keep_lo = f_lo * c_lo, keep_hi = f_hi * c_hi;
    const float add_lo = i_lo * widen_lo(g2), add_hi = i_hi * widen_hi(g2);
    c_lo = keep_lo + add_lo;
    c_hi = keep_hi + add_hi;
    const uint32_t tc2 = ktanh_pair<NANS>(narrow_pair(c_lo, c_hi), tab);
    return narrow_pair(o_lo * widen_lo(tc2), o_hi * widen_hi(tc2));
}

__global__ __launch_bounds__(kBlock) void lstm_cell_kernel(const uint32_t *__restrict__ gates,
                                                           const float2 *__restrict__ c_in,
                                                           float2 *__restrict__ c_out,
                                                           uint32_t *__restrict__ h_out, unsigned T,
                                                           unsigned n_pairs, unsigned H2,
                                                           KtLutPack pack)
{
    const LaneTable tab(pack);
    const unsigned p = blockIdx.x * kBlock + threadIdx.x;
    const bool live = p < n_pairs;
    const unsigned b = live ? p / H2 : 0;
    const unsigned j = live ? p % H2 : 0;
    const unsigned long long row_step = 4ull * n_pairs;  // gate words per time step
    GateOffsets at;
    at.i = (b * 4u * H2 + j) * 4u;  // < 16 * n_pairs <= 2^32 (checked by the caller)
    at.f = at.i + 4u * H2;
    at.g = at.f + 4u * H2;
    at.o = at.g + 4u * H2;

    const unsigned h_at = 4u * p;  // byte offset of this lane's output word inside one step of h

    GateWords stage[kStages];
#pragma unroll
    for (int s = 0; s < kStages; ++s)
        stage[s] = load_gates(gates + s * row_step, at, live && s < (int)T);

    float2 c = float2{0.f, 0.f};
    if (live) c = c_in[p];
    bool suspect = not_finite(c.x) || not_finite(c.y);

    for (unsigned t0 = 0; t0 < T; t0 += kStages) {
#pragma unroll
        for (int s = 0; s < kStages; ++s) {
            const unsigned t = t0 + s;
            if (t < T) {  // uniform over the grid: the table reads below keep every lane enabled
                const GateWords q = stage[s];
                stage[s] = load_gates(gates + (unsigned long long)(t + kStages) * row_step, at,
                                      live && t + kStages < T);
                // NaNs are rare: one test per step for the whole wavefront picks the full rules
                // only when some lane needs them (a wavefront-uniform branch, so that the
                // cross-lane table reads still run with every lane enabled).
                const uint32_t worst = max_pair(max_pair(q.i & kMag2, q.f & kMag2),
                                                max_pair(q.g & kMag2, q.o & kMag2));
                uint32_t h;
                if (__builtin_amdgcn_ballot_w64(suspect || any_nan_pair(worst)) != 0) {
                    h = lstm_step<true>(q, c.x, c.y, tab);
                    suspect = not_finite(c.x) || not_finite(c.y);
                } else {
                    h = lstm_step<false>(q, c.x, c.y, tab);
                }
                if (live) store_stream(h_out + (unsigned long long)t * n_pairs, h_at, h);
            }
        }
    }
    if (live) c_out[p] = c;
}

// ---------------------------------------------------------------------------------------------
// Host side.
int compute_units()
{
    static int cached = 0;  // benign race: every thread computes the same value
    if (cached == 0) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            cus <= 0)
            cus = 256;
        cached = cus;
    }
    return cached;
}

constexpr unsigned kBlocksPerCu = 8;  // resident blocks per compute unit the grid is sized for

ktanh_status_t pack_for(const ktanh_lut_t *lut, bool f32, KtLutPack *pack)
{
    return f32 ? kt_pack_lut_f32(lut, pack) : kt_pack_lut_bf16(lut, pack);
}
ktanh_status_t pack_for(const ktanh_lut64_t *lut, bool f32, KtLutPack *pack)
{
    return f32 ? kt_pack_lut64_f32(lut, pack) : kt_pack_lut64_bf16(lut, pack);
}

template <bool F32, int OP, class Lut>
ktanh_status_t launch_elementwise(const void *in, void *out, size_t n, const Lut *lut,
                                  ktanh_stream_t stream)
{
    constexpr size_t kElem = F32 ? 4 : 2;
    constexpr size_t kPerVec = 16 / kElem;
    if (n == 0) return KT_OK;
    if (in == nullptr || out == nullptr) return KT_ERR_NULL;
    const uintptr_t ain = reinterpret_cast<uintptr_t>(in), aout = reinterpret_cast<uintptr_t>(out);
    if (ain % kElem != 0 || aout % kElem != 0) return KT_ERR_ALIGN;
    if (n > (size_t)1 << 40) return KT_ERR_SHAPE;  // keeps the grid below 2^31 blocks
    KtLutPack pack;
    const ktanh_status_t st = pack_for(lut, F32, &pack);
    if (st != KT_OK) return st;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned max_blocks = (unsigned)compute_units() * kBlocksPerCu;

    if ((ain & 15) == (aout & 15)) {
        size_t head = ((16 - (ain & 15)) & 15) / kElem;
        if (head > n) head = n;
        const size_t nvec = (n - head) / kPerVec;
        const size_t tail = n - head - nvec * kPerVec;
        EdgeArgs edge;
        edge.ein = in;
        edge.eout = out;
        edge.n_total = n;
        edge.n_head = (unsigned)head;
        edge.n_edge = (unsigned)(head + tail);
        const uint4 *vin = reinterpret_cast<const uint4 *>(static_cast<const char *>(in) + head * kElem);
        uint4 *vout = reinterpret_cast<uint4 *>(static_cast<char *>(out) + head * kElem);
        constexpr int kUnroll = (F32 || OP == OP_TANH || OP == OP_TANH64) ? 1 : 2;
        size_t tiles = (nvec + (size_t)kBlock * kUnroll - 1) / ((size_t)kBlock * kUnroll);
        if (tiles == 0) tiles = 1;  // edges only
        if (tiles > 0x7FFFFFFFull) return KT_ERR_SHAPE;
        hipLaunchKernelGGL((stream_kernel<F32, OP, kUnroll>), dim3((unsigned)tiles), dim3(kBlock), 0,
                           s, vin, vout, (unsigned long long)nvec, edge, pack);
    } else {
        const size_t want = (n + kBlock - 1) / kBlock;
        const unsigned blocks = (unsigned)(want < max_blocks ? want : max_blocks);
        hipLaunchKernelGGL((element_kernel<F32, OP>), dim3(blocks), dim3(kBlock), 0, s, in, out,
                           (unsigned long long)n, pack);
    }
    return hipGetLastError() == hipSuccess ? KT_OK : KT_ERR_HIP;
}

}  // namespace

extern "C" ktanh_status_t ktanh_bf16(const uint16_t *in, uint16_t *out, size_t n,
                                     const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    return launch_elementwise<false, OP_TANH>(in, out, n, lut, stream);
}

extern "C" ktanh_status_t ktanh_f32(const uint32_t *in, uint32_t *out, size_t n,
                                    const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    return launch_elementwise<true, OP_TANH>(in, out, n, lut, stream);
}

extern "C" ktanh_status_t ktanh64_bf16(const uint16_t *in, uint16_t *out, size_t n,
                                       const ktanh_lut64_t *lut, ktanh_stream_t stream)
{
    return launch_elementwise<false, OP_TANH64>(in, out, n, lut, stream);
}

extern "C" ktanh_status_t ktanh64_f32(const uint32_t *in, uint32_t *out, size_t n,
                                      const ktanh_lut64_t *lut, ktanh_stream_t stream)
{
    return launch_elementwise<true, OP_TANH64>(in, out, n, lut, stream);
}

extern "C" ktanh_status_t ksigmoid(const uint16_t *in, uint16_t *out, size_t n,
                                   const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    return launch_elementwise<false, OP_SIGMOID>(in, out, n, lut, stream);
}

extern "C" ktanh_status_t kswish(const uint16_t *in, uint16_t *out, size_t n,
                                 const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    return launch_elementwise<false, OP_SWISH>(in, out, n, lut, stream);
}

extern "C" ktanh_status_t kgelu(const uint16_t *in, uint16_t *out, size_t n,
                                const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    return launch_elementwise<false, OP_GELU>(in, out, n, lut, stream);
}

extern "C" ktanh_status_t ksigmoid_f32(const float *in, float *out, size_t n, const ktanh_lut_t *lut,
                                       ktanh_stream_t stream)
{
    return launch_elementwise<true, OP_SIGMOID>(in, out, n, lut, stream);
}

extern "C" ktanh_status_t kswish_f32(const float *in, float *out, size_t n, const ktanh_lut_t *lut,
                                     ktanh_stream_t stream)
{
    return launch_elementwise<true, OP_SWISH>(in, out, n, lut, stream);
}

extern "C" ktanh_status_t kgelu_f32(const float *in, float *out, size_t n, const ktanh_lut_t *lut,
                                    ktanh_stream_t stream)
{
    return launch_elementwise<true, OP_GELU>(in, out, n, lut, stream);
}

extern "C" ktanh_status_t ktanh_f32_to_bf16(const float *in, uint16_t *out, size_t n,
                                            const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    if (n == 0) return KT_OK;
    if (in == nullptr || out == nullptr) return KT_ERR_NULL;
    const uintptr_t ain = reinterpret_cast<uintptr_t>(in), aout = reinterpret_cast<uintptr_t>(out);
    if (ain % 4 != 0 || aout % 2 != 0) return KT_ERR_ALIGN;
    if (n > (size_t)1 << 40) return KT_ERR_SHAPE;
    KtLutPack pack;
    const ktanh_status_t st = kt_pack_lut_bf16(lut, &pack);
    if (st != KT_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);

    size_t head = ((16 - (ain & 15)) & 15) / 4;  // elements until `in` is 16-byte aligned
    if (head > n) head = n;
    if ((aout + 2 * head) % 8 == 0) {
        const size_t nvec = (n - head) / 4;
        const size_t tail = n - head - nvec * 4;
        EdgeArgs edge;
        edge.ein = in;
        edge.eout = out;
        edge.n_total = n;
        edge.n_head = (unsigned)head;
        edge.n_edge = (unsigned)(head + tail);
        size_t tiles = (nvec + (size_t)kBlock * 2 - 1) / ((size_t)kBlock * 2);
        if (tiles == 0) tiles = 1;
        hipLaunchKernelGGL(narrow_stream_kernel, dim3((unsigned)tiles), dim3(kBlock), 0, s,
                           reinterpret_cast<const uint4 *>(in + head),
                           reinterpret_cast<uint2 *>(out + head), (unsigned long long)nvec, edge, pack);
    } else {
        const size_t want = (n + kBlock - 1) / kBlock;
        const size_t max_blocks = (size_t)compute_units() * kBlocksPerCu;
        hipLaunchKernelGGL(narrow_element_kernel, dim3((unsigned)(want < max_blocks ? want : max_blocks)),
                           dim3(kBlock), 0, s, reinterpret_cast<const uint32_t *>(in), out,
                           (unsigned long long)n, pack);
    }
    return hipGetLastError() == hipSuccess ? KT_OK : KT_ERR_HIP;
}

extern "C" ktanh_status_t klstm_cell(const uint16_t *gates, const float *c_in, float *c_out,
                                     uint16_t *h_out, size_t T, size_t B, size_t H,
                                     const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    if (T == 0 || B == 0 || H == 0) return KT_OK;
    if (gates == nullptr || c_in == nullptr || c_out == nullptr || h_out == nullptr)
        return KT_ERR_NULL;
    if (H % 8 != 0) return KT_ERR_SHAPE;
    // sizes: T*B*4H elements must stay far below 2^63, T and H/8 must fit 32 bits
    if (T > 0x7FFFFFFFull || H / 2 > 0xFFFFFFFFull || B > ((size_t)1 << 40) ||
        (B * (H / 8)) > ((size_t)1 << 40) / T)
        return KT_ERR_SHAPE;
    const uintptr_t mis = reinterpret_cast<uintptr_t>(gates) | reinterpret_cast<uintptr_t>(c_in) |
                          reinterpret_cast<uintptr_t>(c_out) | reinterpret_cast<uintptr_t>(h_out);
    if (mis & 15) return KT_ERR_ALIGN;
    KtLutPack pack;
    const ktanh_status_t st = kt_pack_lut_bf16(lut, &pack);
    if (st != KT_OK) return st;

    const unsigned long long n_pairs = (unsigned long long)B * (H / 2);
    if (n_pairs >= (1ull << 28)) return KT_ERR_SHAPE;  // byte offsets inside one step fit 32 bits
    const unsigned long long blocks = (n_pairs + kBlock - 1) / kBlock;
    hipLaunchKernelGGL(lstm_cell_kernel, dim3((unsigned)blocks), dim3(kBlock), 0,
                       static_cast<hipStream_t>(stream), reinterpret_cast<const uint32_t *>(gates),
                       reinterpret_cast<const float2 *>(c_in), reinterpret_cast<float2 *>(c_out),
                       reinterpret_cast<uint32_t *>(h_out), (unsigned)T, (unsigned)n_pairs,
                       (unsigned)(H / 2), pack);
    return hipGetLastError() == hipSuccess ? KT_OK : KT_ERR_HIP;
}
