// Internal to libktanh: the fused LSTM-cell kernel and its launcher, shared by the entry points
// (ktanh_lstm.hip) and by the measurement yardstick (ktanh_probe.hip), so that the yardstick is the
// very same launch with the arithmetic taken out.
#pragma once
#include "ktanh_device.h"

namespace ktanh_device {

// ---------------------------------------------------------------------------------------------
// LSTM cell: each lane owns two neighbouring cells of one batch row (one packed BFloat16 pair per
// gate) and carries their state through all T steps.  The work per cell is about fifty vector
// instructions against ten bytes of traffic, so the kernel wants many wavefronts per SIMD to overlap
// arithmetic with memory rather than wide accesses; a wavefront's loads still cover 256 contiguous
// bytes each.  The steps of one lane are sequential, so the gate words of the next kStages steps are
// already on their way while a step is computed (a ring of register stages): without that the loop
// would pay one full memory latency per step.  The gate non-linearities of a step are formed one step
// early, under the wait for the previous step's K(c').
constexpr int kStages = 4;
constexpr int kCellBlock = 256;  // four wavefronts per block measured best for the short per-step launch

struct GateWords {
    uint32_t i, f, g, o;
};

// Byte offsets of a lane's four gate words inside one time step's [B][4H] gate matrix: 32-bit, so
// that each load is "uniform 64-bit base + 32-bit lane offset" and needs no address arithmetic.
struct GateOffsets {
    unsigned i, f, g, o;
};

// Gate words are read once: the non-temporal hint measured 4-6 % faster than a plain load here.
__device__ __forceinline__ uint32_t load_word(const uint32_t *base, unsigned byte_offset)
{
    return __builtin_nontemporal_load(
        reinterpret_cast<const uint32_t *>(reinterpret_cast<const char *>(base) + byte_offset));
}

__device__ __forceinline__ GateWords load_gates(const uint32_t *step_base, GateOffsets &at)
{
    // The empty statement re-defines the four 32-bit offsets right where they are used, so that
    // each access is selected as "scalar base + 32-bit vector offset"; otherwise their 64-bit
    // extensions are hoisted out of the loop and every access pays a 64-bit vector add.
    asm volatile("" : "+v"(at.i), "+v"(at.f), "+v"(at.g), "+v"(at.o));
    GateWords q;
    q.i = load_word(step_base, at.i);
    q.f = load_word(step_base, at.f);
    q.g = load_word(step_base, at.g);
    q.o = load_word(step_base, at.o);
    return q;
}

// Non-zero where x is an infinity or a NaN.
__device__ __forceinline__ uint32_t not_finite(float x)
{
    return (__float_as_uint(x) & 0x7F800000u) == 0x7F800000u ? 1u : 0u;
}

// The gate non-linearities of one time step for the two cells of a lane.  They depend on the gate
// words alone, not on the state, so they can be formed one step ahead.
struct Acts {
    float i_lo, i_hi, f_lo, f_hi, o_lo, o_hi;
    uint32_t g2;  // K(g) as a BFloat16 pair
};

// NANS = false is the same arithmetic without the NaN rules of K-TanH; it is exact whenever no gate
// word holds a NaN.
template <bool NANS, bool WIDE>
__device__ __forceinline__ Acts activations(const GateWords &q, const LaneTable &tab)
{
    Acts a;
    ksigmoid_f32_pair<NANS, WIDE>(q.i, tab, a.i_lo, a.i_hi);
    ksigmoid_f32_pair<NANS, WIDE>(q.f, tab, a.f_lo, a.f_hi);
    ksigmoid_f32_pair<NANS, WIDE>(q.o, tab, a.o_lo, a.o_hi);
    a.g2 = ktanh_pair<NANS, WIDE>(q.g, tab);
    return a;
}

// c' = (f * c) + (i * g): two products and one sum, each rounded on its own.
__device__ __forceinline__ void advance_state(const Acts &a, float2 &c)
{
    const float keep_lo = a.f_lo * c.x, keep_hi = a.f_hi * c.y;
    const float add_lo = a.i_lo * widen_lo(a.g2), add_hi = a.i_hi * widen_hi(a.g2);
    c.x = keep_lo + add_lo;
    c.y = keep_hi + add_hi;
}

// The state update and the hidden outputs of one step from its activations, with the full NaN rules
// (exact for any input).
template <bool WIDE>
__device__ __forceinline__ uint32_t finish_step_checked(const Acts &a, float2 &c, const LaneTable &tab)
{
    advance_state(a, c);
    const uint32_t tc2 = ktanh_pair<true, WIDE>(narrow_pair(c.x, c.y), tab);
    return narrow_pair(a.o_lo * widen_lo(tc2), a.o_hi * widen_hi(tc2));
}

// True for the whole wavefront when some lane holds a NaN in one of its four gate words.
__device__ __forceinline__ bool gates_hold_nan(const GateWords &q)
{
    const uint32_t worst = max_pair(max_pair(q.i & kMag2, q.f & kMag2),
                                    max_pair(q.g & kMag2, q.o & kMag2));
    return __builtin_amdgcn_ballot_w64(nan_bits_pair(worst) != 0u) != 0;
}

// One time step, and the activations of the next one.  `a` holds the activations of this step and
// is replaced by those of the step whose gate words are `next`; `a_checked` says (for the whole
// wavefront) whether `a` was formed under the NaN rules, i.e. may hold a NaN.
//
// The steps of a lane form one dependent chain (state -> K(state) -> output), and each K costs a
// round trip through the cross-lane unit.  With only four wavefronts per SIMD that latency is not
// hidden by other wavefronts, so it is hidden inside the wavefront: the table reads for K(c') are
// put in flight, the next step's activations (four independent K evaluations) are formed while they
// travel, and only then is K(c') finished.
//
// NaNs are rare: the fast path drops the NaN rules and runs only when no lane of the wavefront needs
// them (wavefront-uniform branches, so that the cross-lane table reads still run with every lane
// enabled).  `suspect` is a per-lane flag word (non-zero = this lane's state may not be finite);
// always_checked: the caller's table lets |K| exceed 1, so the state may overflow on the way.
template <bool WIDE>
__device__ __forceinline__ uint32_t step_and_look_ahead(Acts &a, bool &a_checked, const GateWords &next,
                                                        float2 &c, uint32_t &suspect,
                                                        uint32_t always_checked, const LaneTable &tab)
{
    const bool next_checked = gates_hold_nan(next);
    const bool now_checked = a_checked || __builtin_amdgcn_ballot_w64(suspect != 0u) != 0;
    uint32_t h;
    if (!now_checked && !next_checked) {
        // exact here: no gate is a NaN, the incoming state is finite and |K| <= 1, so the state
        // stays finite (|c'| <= |c| + 1)
        advance_state(a, c);
        const uint32_t cb = narrow_pair(c.x, c.y);
        const uint32_t mag2 = cb & kMag2;
        const SlotPair sp = fetch_slots<WIDE>(mag2, tab);
        const Acts ahead = activations<false, WIDE>(next, tab);
        const uint32_t tc2 = bitsel(kMag2, finish_mag_pair<WIDE>(mag2, sp), cb);
        h = narrow_pair(a.o_lo * widen_lo(tc2), a.o_hi * widen_hi(tc2));
        a = ahead;
    } else {
        h = finish_step_checked<WIDE>(a, c, tab);
        suspect = always_checked | not_finite(c.x) | not_finite(c.y);
        a = activations<true, WIDE>(next, tab);
    }
    a_checked = next_checked;
    return h;
}

// The last step of a call: no next gate words to look at.
template <bool WIDE>
__device__ __forceinline__ uint32_t last_step(const Acts &a, float2 &c, const LaneTable &tab)
{
    return finish_step_checked<WIDE>(a, c, tab);
}

// ARITH = false is the measurement form of the kernel: the same loads, stores, waits and loop with
// the arithmetic taken out.  A step's output word is then the XOR of its four gate words and the
// bits of the lane's first state value (so that no load can be dropped), formed one step ahead like
// the activations, and the state passes through unchanged.
__device__ __forceinline__ uint32_t fold(const GateWords &q) { return q.i ^ q.f ^ q.g ^ q.o; }

template <bool WIDE, bool ARITH>
__device__ __forceinline__ uint32_t one_step(Acts &a, bool &a_checked, const GateWords &next, float2 &c,
                                             uint32_t &suspect, uint32_t always_checked,
                                             const LaneTable &tab)
{
    if constexpr (ARITH) {
        return step_and_look_ahead<WIDE>(a, a_checked, next, c, suspect, always_checked, tab);
    } else {
        const uint32_t h = a.g2 ^ __float_as_uint(c.x);
        a.g2 = fold(next);
        return h;
    }
}

template <bool WIDE, bool ARITH>
__device__ __forceinline__ uint32_t final_step(const Acts &a, float2 &c, const LaneTable &tab)
{
    if constexpr (ARITH) return last_step<WIDE>(a, c, tab);
    else return a.g2 ^ __float_as_uint(c.x);
}

template <bool WIDE, bool ARITH>
__global__ __launch_bounds__(kCellBlock) void lstm_cell_kernel(const uint32_t *__restrict__ gates,
                                                           const float2 *c_in, float2 *c_out,  // may be equal
                                                           uint32_t *__restrict__ h_out, unsigned T,
                                                           unsigned n_pairs, unsigned H2,
                                                           unsigned always_checked, KtLutPack pack)
{
    const LaneTable tab(pack);
    const unsigned p = blockIdx.x * kCellBlock + threadIdx.x;
    const bool live = p < n_pairs;
    // Lanes past the end work on pair 0 and store nothing: every lane then issues every load, with
    // no branch around it, which lets each step wait for exactly its own gate words (a load that
    // only some paths issue makes the wait cover everything in flight).
    const unsigned p_read = live ? p : 0;
    const unsigned b = p_read / H2;
    const unsigned j = p_read % H2;
    const unsigned long long row_step = 4ull * n_pairs;  // gate words per time step
    GateOffsets at;
    at.i = (b * 4u * H2 + j) * 4u;  // < 16 * n_pairs <= 2^32 (checked by the caller)
    at.f = at.i + 4u * H2;
    at.g = at.f + 4u * H2;
    at.o = at.g + 4u * H2;
    const unsigned h_at = 4u * p;  // byte offset of this lane's output word inside one step of h

    float2 c = c_in[p_read];  // first in the queue: its wait leaves the gate words in flight
    GateWords stage[kStages];
    const uint32_t *ahead = gates;  // the next step to fetch
    uint32_t *h_row = h_out;        // the next step to store
    unsigned t = 0;

    const bool ring = T >= 2u * kStages;
#pragma unroll
    for (int s = 0; s < kStages; ++s) {
        stage[s] = GateWords{0u, 0u, 0u, 0u};
        if (ring || s < (int)T) {  // uniform over the grid
            stage[s] = load_gates(ahead, at);
            ahead += row_step;
        }
    }
    uint32_t suspect = always_checked | not_finite(c.x) | not_finite(c.y);
    // the activations of step 0, under the full rules (once per call)
    Acts a = Acts{};
    if constexpr (ARITH) a = activations<true, WIDE>(stage[0], tab);
    else a.g2 = fold(stage[0]);
    bool a_checked = true;

    if (ring) {
        // Steady state: stage s holds the gate words of the current step, stage s + 1 those of the
        // next; each stage is refilled right after the step that consumed it, in place (the refill
        // follows the step's last use of the old words, so that no register copies -- which would
        // have to wait for every load in flight -- are needed at the end of the body).
        for (; t + 2u * kStages <= T; t += kStages) {
#pragma unroll
            for (int s = 0; s < kStages; ++s) {
                const uint32_t h = one_step<WIDE, ARITH>(a, a_checked, stage[(s + 1) % kStages], c,
                                                         suspect, always_checked, tab);
                if (live) store_stream(h_row, h_at, h);
                h_row += n_pairs;
                stage[s] = load_gates(ahead, at);
                ahead += row_step;
            }
        }
    }

    // The last steps (fewer than 2 * kStages): stage k % kStages holds step t + k.  Written out step
    // by step with the stages named statically, like the steady loop: moving the ring up through
    // register copies instead would make every one of these steps wait for all loads in flight,
    // a full memory latency each.  All conditions are uniform over the grid.
#pragma unroll
    for (int k = 0; k < 2 * kStages - 1; ++k) {
        if (t + k < T) {
            constexpr int kRing = kStages;
            const int s = k % kRing;
            uint32_t h;
            if (t + k + 1 < T)
                h = one_step<WIDE, ARITH>(a, a_checked, stage[(s + 1) % kRing], c, suspect,
                                          always_checked, tab);
            else
                h = final_step<WIDE, ARITH>(a, c, tab);
            if (live) store_stream(h_row, h_at, h);
            h_row += n_pairs;
            if (k < kRing && t + k + kRing < T) {
                stage[s] = load_gates(ahead, at);
                ahead += row_step;
            }
        }
    }
    if (live) c_out[p] = c;
}

inline ktanh_status_t pack_cell(const ktanh_lut_t *lut, KtLutPack *pack, bool *within_unit)
{
    return kt_pack_lut_bf16(lut, pack, within_unit);
}
inline ktanh_status_t pack_cell(const ktanh_lut64_t *lut, KtLutPack *pack, bool *within_unit)
{
    return kt_pack_lut64_bf16(lut, pack, within_unit);
}

template <bool WIDE, bool ARITH = true, class Lut>
ktanh_status_t launch_cell(const uint16_t *gates, const float *c_in, float *c_out, uint16_t *h_out,
                           size_t T, size_t B, size_t H, const Lut *lut, ktanh_stream_t stream)
{
    if (T == 0 || B == 0 || H == 0) return KT_OK;
    if (gates == nullptr || c_in == nullptr || c_out == nullptr || h_out == nullptr)
        return KT_ERR_NULL;
    if (H % 8 != 0) return KT_ERR_SHAPE;
    // one time step holds fewer than 2^28 lane pairs (byte offsets inside a step fit 32 bits), and
    // T*B*4H elements stay far below 2^63; every bound is tested by division, so nothing wraps
    if (T > 0x7FFFFFFFull || B >= ((size_t)1 << 28) || H >= ((size_t)1 << 29) ||
        B > (((size_t)1 << 28) - 1) / (H / 2))
        return KT_ERR_SHAPE;
    // the kernel moves BFloat16 pairs (4 bytes) and Float32 pairs (8 bytes)
    const uintptr_t words = reinterpret_cast<uintptr_t>(gates) | reinterpret_cast<uintptr_t>(h_out);
    const uintptr_t states = reinterpret_cast<uintptr_t>(c_in) | reinterpret_cast<uintptr_t>(c_out);
    if ((words & 3) || (states & 7)) return KT_ERR_ALIGN;
    KtLutPack pack;
    bool within_unit = true;
    const ktanh_status_t st = pack_cell(lut, &pack, &within_unit);
    if (st != KT_OK) return st;

    const unsigned long long n_pairs = (unsigned long long)B * (H / 2);  // < 2^28, checked above
    const unsigned long long blocks = (n_pairs + kCellBlock - 1) / kCellBlock;
    return launch_checked(lstm_cell_kernel<WIDE, ARITH>, (unsigned)blocks, kCellBlock, stream,
                          reinterpret_cast<const uint32_t *>(gates),
                          reinterpret_cast<const float2 *>(c_in), reinterpret_cast<float2 *>(c_out),
                          reinterpret_cast<uint32_t *>(h_out), (unsigned)T, (unsigned)n_pairs,
                          (unsigned)(H / 2), within_unit ? 0u : 1u, pack);
}

}  // namespace ktanh_device
