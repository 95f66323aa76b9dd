// libktanh: the element-wise streaming kernels (K-TanH on BFloat16 / Float32, 32 or 64 intervals,
// Sigmoid / Swish / GELU on both formats, Float32 -> BFloat16 K-TanH) and their entry points.
//
// Shape of every kernel: a pure HBM stream.  Each lane moves 128 bits per access (8 BFloat16 or
// 4 Float32), a wavefront covers 1 KiB per access, and every block handles one tile and exits.
#include "ktanh_device.h"

using namespace ktanh_device;

namespace {

static_assert(kBlock == 64, "the loose elements (fewer than 64) are taken by the one wavefront of block 0");

// ---------------------------------------------------------------------------------------------
// Element-wise streaming kernel over `nvec` 128-bit vectors plus up to `n_edge` loose elements.
//   vin, vout : the body (nvec vectors); vout is 16-byte aligned, vin too unless IN_UNALIGNED
//   skew      : index of vout's first vector inside its 1 KiB group (0..63).  Tiles are cut at
//               1 KiB boundaries of `out`, the first one short: a wavefront's store then never
//               shares a cache line with its neighbour's (a body that starts 16 bytes into a line
//               otherwise runs 17 % slower on the same tensor)
//   ein, eout : the whole tensor as elements; edge element k (k < n_head) is element k, edge
//               element k >= n_head is element n_total - n_edge + k (the ragged tail)
// F32 selects the Float32 operations, else the BFloat16 ones.
struct EdgeArgs {
    const void *ein;
    void *eout;
    unsigned long long n_total;
    unsigned n_head;
    unsigned n_edge;  // head + tail elements, < 64
    unsigned skew;
};

template <bool F32, int OP, bool WIDE>
__device__ __forceinline__ uint4 apply_vec(uint4 v, const LaneTable &tab)
{
    if constexpr (F32) return apply_vec_f32<OP, WIDE>(v, tab);
    else return apply_vec_bf16<OP, WIDE>(v, tab);
}

// IN_UNALIGNED: `in` and `out` disagree modulo 16 bytes; the stores stay aligned, the loads are
// 16-byte loads from element-aligned addresses (2.2x faster than one element per lane).
template <bool F32, int OP, bool WIDE, bool IN_UNALIGNED>
__global__ __launch_bounds__(kBlock) void stream_kernel(const uint4 *vin, uint4 *vout,  // may be equal
                                                        unsigned long long nvec, EdgeArgs edge,
                                                        KtLutPack pack)
{
    const LaneTable tab(pack);

    // One vector per lane, one tile of kBlock vectors per block, no loop: fresh blocks keep loads and
    // stores of different tiles overlapped, which a grid-stride loop over the same tiles does not
    // (measured: 6.5 against 6.0 TB/s on a 537 MB stream).  Single-wavefront blocks measured best for
    // every operation (5 % over 256-thread blocks on a 105 MB tensor, two vectors per lane another
    // 3-5 % slower): with 32 independent wavefronts per compute unit even GELU's arithmetic hides
    // under the stream.
    const unsigned long long slot = (unsigned long long)blockIdx.x * kBlock + threadIdx.x;
    const unsigned long long at = slot - edge.skew;
    const bool live_vec = slot >= edge.skew && at < nvec;
    uint4 v = uint4{0u, 0u, 0u, 0u};
    if (live_vec) {
        if constexpr (IN_UNALIGNED) v = load_stream_unaligned(reinterpret_cast<const char *>(vin) + 16 * at);
        else v = load_stream(vin + at);
    }
    v = apply_vec<F32, OP, WIDE>(v, tab);
    if (live_vec) store_stream(vout + at, v);

    // Loose elements before and after the aligned body: first wavefront of block 0.
    if (edge.n_edge != 0 && blockIdx.x == 0) {  // uniform over the block
        const unsigned k = threadIdx.x;
        const bool live = k < edge.n_edge;
        const unsigned long long i =
            k < edge.n_head ? k : edge.n_total - edge.n_edge + k;
        uint32_t x = 0;
        if constexpr (F32) {
            if (live) x = static_cast<const uint32_t *>(edge.ein)[i];
            x = apply_f32_one<OP, WIDE>(x, tab);
            if (live) static_cast<uint32_t *>(edge.eout)[i] = x;
        } else {
            if (live) x = static_cast<const uint16_t *>(edge.ein)[i];
            x = apply_pair<OP, WIDE>(x, tab);
            if (live) static_cast<uint16_t *>(edge.eout)[i] = (uint16_t)x;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Float32 in, BFloat16 out: round to nearest even (v_cvt_pk_bf16_f32), then K-TanH.  Each lane
// reads one 128-bit vector (4 Float32) and writes one 64-bit one.
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

// Tiles are cut at 512-byte boundaries of `out` (edge.skew, as in stream_kernel); IN_UNALIGNED as there.
template <bool IN_UNALIGNED>
__global__ __launch_bounds__(kBlock) void narrow_stream_kernel(const uint4 *__restrict__ vin,
                                                               uint2 *__restrict__ vout,
                                                               unsigned long long nvec,
                                                               EdgeArgs edge, KtLutPack pack)
{
    const LaneTable tab(pack);
    const unsigned long long slot = (unsigned long long)blockIdx.x * kBlock + threadIdx.x;
    const unsigned long long at = slot - edge.skew;
    const bool live_vec = slot >= edge.skew && at < nvec;
    uint4 v = uint4{0u, 0u, 0u, 0u};
    if (live_vec) {
        if constexpr (IN_UNALIGNED) v = load_stream_unaligned(reinterpret_cast<const char *>(vin) + 16 * at);
        else v = load_stream(vin + at);
    }
    const uint2 o = narrow_ktanh_vec(v, tab);
    if (live_vec) store_stream(vout + at, o);

    if (edge.n_edge != 0 && blockIdx.x == 0) {  // uniform over the block
        const unsigned k = threadIdx.x;
        const bool live = k < edge.n_edge;
        const unsigned long long i = k < edge.n_head ? k : edge.n_total - edge.n_edge + k;
        uint32_t x = 0;
        if (live) x = static_cast<const uint32_t *>(edge.ein)[i];
        x = ktanh_pair(narrow_pair(__uint_as_float(x), 0.0f), tab);
        if (live) static_cast<uint16_t *>(edge.eout)[i] = (uint16_t)x;
    }
}

// ---------------------------------------------------------------------------------------------
// Host side.
ktanh_status_t pack_for(const ktanh_lut_t *lut, bool f32, KtLutPack *pack)
{
    return f32 ? kt_pack_lut_f32(lut, pack) : kt_pack_lut_bf16(lut, pack);
}
ktanh_status_t pack_for(const ktanh_lut64_t *lut, bool f32, KtLutPack *pack)
{
    return f32 ? kt_pack_lut64_f32(lut, pack) : kt_pack_lut64_bf16(lut, pack);
}

constexpr bool is_wide(const ktanh_lut_t *) { return false; }
constexpr bool is_wide(const ktanh_lut64_t *) { return true; }

template <bool F32, int OP, class Lut>
ktanh_status_t launch_elementwise(const void *in, void *out, size_t n, const Lut *lut,
                                  ktanh_stream_t stream)
{
    constexpr bool WIDE = is_wide(static_cast<const Lut *>(nullptr));
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

    // Peel elements until `out` reaches a 16-byte boundary; the body's loads are aligned too when
    // `in` is congruent to `out` modulo 16, else they are unaligned 16-byte loads.
    size_t head = ((16 - (aout & 15)) & 15) / kElem;
    if (head > n) head = n;
    const size_t nvec = (n - head) / kPerVec;
    const size_t tail = n - head - nvec * kPerVec;
    const uint4 *vin = reinterpret_cast<const uint4 *>(static_cast<const char *>(in) + head * kElem);
    uint4 *vout = reinterpret_cast<uint4 *>(static_cast<char *>(out) + head * kElem);
    EdgeArgs edge;
    edge.ein = in;
    edge.eout = out;
    edge.n_total = n;
    edge.n_head = (unsigned)head;
    edge.n_edge = (unsigned)(head + tail);
    edge.skew = (unsigned)((reinterpret_cast<uintptr_t>(vout) / 16) % kBlock);
    size_t tiles = (nvec + edge.skew + kBlock - 1) / kBlock;
    if (tiles == 0) tiles = 1;  // edges only
    if (tiles > 0x7FFFFFFFull) return KT_ERR_SHAPE;
    if ((ain & 15) == (aout & 15))
        return launch_checked(stream_kernel<F32, OP, WIDE, false>, (unsigned)tiles, kBlock, stream,
                              vin, vout, (unsigned long long)nvec, edge, pack);
    return launch_checked(stream_kernel<F32, OP, WIDE, true>, (unsigned)tiles, kBlock, stream, vin,
                          vout, (unsigned long long)nvec, edge, pack);
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
    return launch_elementwise<false, OP_TANH>(in, out, n, lut, stream);
}

extern "C" ktanh_status_t ktanh64_f32(const uint32_t *in, uint32_t *out, size_t n,
                                      const ktanh_lut64_t *lut, ktanh_stream_t stream)
{
    return launch_elementwise<true, OP_TANH>(in, out, n, lut, stream);
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

extern "C" ktanh_status_t ksigmoid64(const uint16_t *in, uint16_t *out, size_t n,
                                     const ktanh_lut64_t *lut, ktanh_stream_t stream)
{
    return launch_elementwise<false, OP_SIGMOID>(in, out, n, lut, stream);
}

extern "C" ktanh_status_t kswish64(const uint16_t *in, uint16_t *out, size_t n,
                                   const ktanh_lut64_t *lut, ktanh_stream_t stream)
{
    return launch_elementwise<false, OP_SWISH>(in, out, n, lut, stream);
}

extern "C" ktanh_status_t kgelu64(const uint16_t *in, uint16_t *out, size_t n,
                                  const ktanh_lut64_t *lut, ktanh_stream_t stream)
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

    size_t head = ((8 - (aout & 7)) & 7) / 2;  // elements until `out` is 8-byte aligned
    if (head > n) head = n;
    const size_t nvec = (n - head) / 4;
    const size_t tail = n - head - nvec * 4;
    EdgeArgs edge;
    edge.ein = in;
    edge.eout = out;
    edge.n_total = n;
    edge.n_head = (unsigned)head;
    edge.n_edge = (unsigned)(head + tail);
    edge.skew = (unsigned)((reinterpret_cast<uintptr_t>(out + head) / 8) % kBlock);
    size_t tiles = (nvec + edge.skew + kBlock - 1) / kBlock;
    if (tiles == 0) tiles = 1;
    if (tiles > 0x7FFFFFFFull) return KT_ERR_SHAPE;
    const uint4 *vin = reinterpret_cast<const uint4 *>(in + head);
    uint2 *vout = reinterpret_cast<uint2 *>(out + head);
    if (reinterpret_cast<uintptr_t>(vin) % 16 == 0)
        return launch_checked(narrow_stream_kernel<false>, (unsigned)tiles, kBlock, stream, vin, vout,
                              (unsigned long long)nvec, edge, pack);
    return launch_checked(narrow_stream_kernel<true>, (unsigned)tiles, kBlock, stream, vin, vout,
                          (unsigned long long)nvec, edge, pack);
}

extern "C" ktanh_status_t ksigmoid64_f32(const float *in, float *out, size_t n,
                                         const ktanh_lut64_t *lut, ktanh_stream_t stream)
{
    return launch_elementwise<true, OP_SIGMOID>(in, out, n, lut, stream);
}

extern "C" ktanh_status_t kswish64_f32(const float *in, float *out, size_t n,
                                       const ktanh_lut64_t *lut, ktanh_stream_t stream)
{
    return launch_elementwise<true, OP_SWISH>(in, out, n, lut, stream);
}

extern "C" ktanh_status_t kgelu64_f32(const float *in, float *out, size_t n,
                                      const ktanh_lut64_t *lut, ktanh_stream_t stream)
{
    return launch_elementwise<true, OP_GELU>(in, out, n, lut, stream);
}

extern "C" ktanh_status_t ktanh_stream_copy(const uint16_t *in, uint16_t *out, size_t n,
                                            ktanh_stream_t stream)
{
    return launch_elementwise<false, OP_COPY>(in, out, n, static_cast<const ktanh_lut_t *>(nullptr), stream);
}
