// Internal to libktanh: the element-wise streaming kernel and its launcher, shared by the entry
// points (ktanh_stream.hip) and by the measurement yardsticks (ktanh_probe.hip), so that a yardstick
// is the very same launch with the arithmetic taken out.
#pragma once
#include "ktanh_device.h"

namespace ktanh_device {

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
//
// The arguments every wavefront needs before it can issue its load (vin, vout, nvec, skew, n_edge)
// come first and are scalars: the library is compiled so that the leading scalar arguments of a
// kernel arrive preloaded in registers, which saves each of the many short-lived wavefronts a
// round trip to the argument buffer (measured: 0.7-1 % on 100-500 MB tensors).
struct EdgeArgs {
    const void *ein;
    void *eout;
    unsigned long long n_total;
    unsigned n_head;
};

template <bool F32, int OP, bool WIDE, class Tab>
__device__ __forceinline__ uint4 apply_vec(uint4 v, const Tab &tab)
{
    if constexpr (F32) return apply_vec_f32<OP, WIDE>(v, tab);
    else return apply_vec_bf16<OP, WIDE>(v, tab);
}

// IN_UNALIGNED: `in` and `out` disagree modulo 16 bytes; the stores stay aligned, the loads are
// 16-byte loads from element-aligned addresses (2.2x faster than one element per lane).
template <bool F32, int OP, bool WIDE, bool IN_UNALIGNED>
__global__ __launch_bounds__(kBlock) void stream_kernel(const uint4 *vin, uint4 *vout,  // may be equal
                                                        unsigned long long nvec, unsigned skew,
                                                        unsigned n_edge /* head + tail, < 64 */,
                                                        unsigned whole, unsigned lg_seg,  // TileOrder
                                                        EdgeArgs edge, typename TableOf<OP>::Pack pack)
{
    const typename TableOf<OP>::Lane tab(pack);

    // One vector per lane, one tile of kBlock vectors per block, no loop: fresh blocks keep loads and
    // stores of different tiles overlapped, which a grid-stride loop over the same tiles does not
    // (measured: 6.5 against 6.0 TB/s on a 537 MB stream).  Single-wavefront blocks measured best for
    // every operation (5 % over 256-thread blocks on a 105 MB tensor, two vectors per lane another
    // 3-5 % slower): with 32 independent wavefronts per compute unit even GELU's arithmetic hides
    // under the stream.
    const unsigned long long slot =
        (unsigned long long)tile_of_block(blockIdx.x, whole, lg_seg) * kBlock + threadIdx.x;
    const unsigned long long at = slot - skew;
    const bool live_vec = slot >= skew && at < nvec;
    uint4 v = uint4{0u, 0u, 0u, 0u};
    if (live_vec) {
        if constexpr (IN_UNALIGNED) v = load_stream_unaligned(reinterpret_cast<const char *>(vin) + 16 * at);
        else v = load_stream(vin + at);
    }
    v = apply_vec<F32, OP, WIDE>(v, tab);
    if (live_vec) store_stream(vout + at, v);

    // Loose elements before and after the aligned body: first wavefront of block 0.
    if (n_edge != 0 && blockIdx.x == 0) {  // uniform over the block
        const unsigned k = threadIdx.x;
        const bool live = k < n_edge;
        const unsigned long long i =
            k < edge.n_head ? k : edge.n_total - n_edge + k;
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
// Host side.
inline ktanh_status_t pack_for(const ktanh_lut_t *lut, bool f32, KtLutPack *pack)
{
    return f32 ? kt_pack_lut_f32(lut, pack) : kt_pack_lut_bf16(lut, pack);
}
inline ktanh_status_t pack_for(const ktanh_lut64_t *lut, bool f32, KtLutPack *pack)
{
    return f32 ? kt_pack_lut64_f32(lut, pack) : kt_pack_lut64_bf16(lut, pack);
}

// The Taylor polynomials have one fixed table, formed once per process; the caller's table argument
// is not used.
inline ktanh_status_t pack_for(const ktanh_lut_t *, bool, KtTaylorPack *pack)
{
    static const KtTaylorPack table = [] {
        KtTaylorPack t;
        kt_pack_taylor(&t);
        return t;
    }();
    *pack = table;
    return KT_OK;
}

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
    typename TableOf<OP>::Pack pack;
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
    const unsigned n_edge = (unsigned)(head + tail);
    const unsigned skew = (unsigned)((reinterpret_cast<uintptr_t>(vout) / 16) % kBlock);
    size_t tiles = (nvec + skew + kBlock - 1) / kBlock;
    if (tiles == 0) tiles = 1;  // edges only
    if (tiles > kMaxTiles) return KT_ERR_SHAPE;
    const TileOrder order = tile_order_for(tiles);
    if ((ain & 15) == (aout & 15))
        return launch_checked(stream_kernel<F32, OP, WIDE, false>, (unsigned)tiles, kBlock, stream,
                              vin, vout, (unsigned long long)nvec, skew, n_edge, order.whole,
                              order.lg_seg, edge, pack);
    return launch_checked(stream_kernel<F32, OP, WIDE, true>, (unsigned)tiles, kBlock, stream, vin,
                          vout, (unsigned long long)nvec, skew, n_edge, order.whole, order.lg_seg, edge,
                          pack);
}

}  // namespace ktanh_device
