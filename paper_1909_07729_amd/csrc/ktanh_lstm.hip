// libktanh: the fused LSTM-cell element-wise kernel and its entry point.
#include "ktanh_device.h"

using namespace ktanh_device;

namespace {

// ---------------------------------------------------------------------------------------------
// LSTM cell: each lane owns two neighbouring cells of one batch row (one packed BFloat16 pair per
// gate) and carries their state through all T steps.  The work per cell is about fifty vector
// instructions against ten bytes of traffic, so the kernel wants many wavefronts per SIMD to overlap
// arithmetic with memory rather than wide accesses; a wavefront's loads still cover 256 contiguous
// bytes each.  The steps of one lane are sequential, so the gate words of the next kStages steps are
// already on their way while a step is computed (a ring of register stages): without that the loop
// would pay one full memory latency per step.
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

// One time step for the two cells of a lane: updates their state, returns the two hidden outputs.
// NANS = false is the same arithmetic without the NaN rules of K-TanH; it is exact whenever no gate
// is NaN, the incoming state is finite and the table keeps |K| <= 1 (the state then stays finite:
// |c'| <= |c| + 1).
template <bool NANS, bool WIDE>
__device__ __forceinline__ uint32_t lstm_step(const GateWords &q, float &c_lo, float &c_hi,
                                              const LaneTable &tab)
{
    // One gate after the other: putting all eight table reads of the four gates in flight first
    // measured 10 % slower (the four wavefronts of a SIMD then stall and resume in step).
    float i_lo, i_hi, f_lo, f_hi, o_lo, o_hi;
    ksigmoid_f32_pair<NANS, WIDE>(q.i, tab, i_lo, i_hi);
    ksigmoid_f32_pair<NANS, WIDE>(q.f, tab, f_lo, f_hi);
    ksigmoid_f32_pair<NANS, WIDE>(q.o, tab, o_lo, o_hi);
    const uint32_t g2 = ktanh_pair<NANS, WIDE>(q.g, tab);
    // c' = (f * c) + (i * g): two products and one sum, each rounded on its own
    const float keep_lo = f_lo * c_lo, keep_hi = f_hi * c_hi;
    const float add_lo = i_lo * widen_lo(g2), add_hi = i_hi * widen_hi(g2);
    c_lo = keep_lo + add_lo;
    c_hi = keep_hi + add_hi;
    const uint32_t tc2 = ktanh_pair<NANS, WIDE>(narrow_pair(c_lo, c_hi), tab);
    return narrow_pair(o_lo * widen_lo(tc2), o_hi * widen_hi(tc2));
}

// NaNs are rare: one test per step for the whole wavefront picks the full rules only when some
// lane needs them (a wavefront-uniform branch, so that the cross-lane table reads still run with
// every lane enabled).  always_checked: the caller's table lets |K| exceed 1, so the state may
// overflow on the way.
// `suspect` is a per-lane flag word (non-zero = this lane's state may not be finite), kept as a
// number so that it joins the gate test with one OR.
template <bool WIDE>
__device__ __forceinline__ uint32_t guarded_step(const GateWords &q, float2 &c, uint32_t &suspect,
                                                 uint32_t always_checked, const LaneTable &tab)
{
    const uint32_t worst = max_pair(max_pair(q.i & kMag2, q.f & kMag2),
                                    max_pair(q.g & kMag2, q.o & kMag2));
    uint32_t h;
    if (__builtin_amdgcn_ballot_w64((nan_bits_pair(worst) | suspect) != 0u) != 0) {
        h = lstm_step<true, WIDE>(q, c.x, c.y, tab);
        suspect = always_checked | not_finite(c.x) | not_finite(c.y);
    } else {
        h = lstm_step<false, WIDE>(q, c.x, c.y, tab);
    }
    return h;
}

template <bool WIDE>
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
    uint32_t suspect;

    if (T >= 2u * kStages) {
#pragma unroll
        for (int s = 0; s < kStages; ++s, ahead += row_step) stage[s] = load_gates(ahead, at);
        suspect = always_checked | not_finite(c.x) | not_finite(c.y);
        // Steady state: each stage is refilled right after the step that consumed it, in place
        // (the refill follows the step's last use of the old words, so that no register copies --
        // which would have to wait for every load in flight -- are needed at the end of the body).
        for (; t + 2u * kStages <= T; t += kStages) {
#pragma unroll
            for (int s = 0; s < kStages; ++s) {
                const uint32_t h = guarded_step<WIDE>(stage[s], c, suspect, always_checked, tab);
                if (live) store_stream(h_row, h_at, h);
                h_row += n_pairs;
                stage[s] = load_gates(ahead, at);
                ahead += row_step;
            }
        }
    } else {
#pragma unroll
        for (int s = 0; s < kStages; ++s) {
            stage[s] = GateWords{0u, 0u, 0u, 0u};
            if (s < (int)T) {  // uniform over the grid
                stage[s] = load_gates(ahead, at);
                ahead += row_step;
            }
        }
        suspect = always_checked | not_finite(c.x) | not_finite(c.y);
    }

    // The last steps (fewer than 2 * kStages): stage[0] is the current one, the ring moves up.
    const uint32_t *const gates_end = gates + (unsigned long long)T * row_step;
    for (; t < T; ++t) {
        const uint32_t h = guarded_step<WIDE>(stage[0], c, suspect, always_checked, tab);
        if (live) store_stream(h_row, h_at, h);
        h_row += n_pairs;
#pragma unroll
        for (int s = 0; s + 1 < kStages; ++s) stage[s] = stage[s + 1];
        stage[kStages - 1] = GateWords{0u, 0u, 0u, 0u};
        if (ahead != gates_end) {  // uniform over the grid
            stage[kStages - 1] = load_gates(ahead, at);
            ahead += row_step;
        }
    }
    if (live) c_out[p] = c;
}

ktanh_status_t pack_cell(const ktanh_lut_t *lut, KtLutPack *pack, bool *within_unit)
{
    return kt_pack_lut_bf16(lut, pack, within_unit);
}
ktanh_status_t pack_cell(const ktanh_lut64_t *lut, KtLutPack *pack, bool *within_unit)
{
    return kt_pack_lut64_bf16(lut, pack, within_unit);
}

template <bool WIDE, class Lut>
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
    return launch_checked(lstm_cell_kernel<WIDE>, (unsigned)blocks, kCellBlock, stream,
                          reinterpret_cast<const uint32_t *>(gates),
                          reinterpret_cast<const float2 *>(c_in), reinterpret_cast<float2 *>(c_out),
                          reinterpret_cast<uint32_t *>(h_out), (unsigned)T, (unsigned)n_pairs,
                          (unsigned)(H / 2), within_unit ? 0u : 1u, pack);
}

}  // namespace

extern "C" ktanh_status_t klstm_cell(const uint16_t *gates, const float *c_in, float *c_out,
                                     uint16_t *h_out, size_t T, size_t B, size_t H,
                                     const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    return launch_cell<false>(gates, c_in, c_out, h_out, T, B, H, lut, stream);
}

extern "C" ktanh_status_t klstm_cell64(const uint16_t *gates, const float *c_in, float *c_out,
                                       uint16_t *h_out, size_t T, size_t B, size_t H,
                                       const ktanh_lut64_t *lut, ktanh_stream_t stream)
{
    return launch_cell<true>(gates, c_in, c_out, h_out, T, B, H, lut, stream);
}
