// libktanh: the element-wise streaming kernels (K-TanH on BFloat16 / Float32, 32 or 64 intervals,
// Sigmoid / Swish / GELU on both formats, Float32 -> BFloat16 K-TanH) and their entry points.
//
// Shape of every kernel: a pure HBM stream.  Each lane moves 128 bits per access (8 BFloat16 or
// 4 Float32), a wavefront covers 1 KiB per access, and every block handles one tile and exits.
#include "ktanh_stream_impl.h"

using namespace ktanh_device;

namespace {

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

// Tiles are cut at 512-byte boundaries of `out` (skew, as in stream_kernel); IN_UNALIGNED as there.
template <bool IN_UNALIGNED>
__global__ __launch_bounds__(kBlock) void narrow_stream_kernel(const uint4 *__restrict__ vin,
                                                               uint2 *__restrict__ vout,
                                                               unsigned long long nvec,
                                                               unsigned skew, unsigned n_edge,
                                                               EdgeArgs edge, KtLutPack pack)
{
    const LaneTable tab(pack);
    const unsigned long long slot = (unsigned long long)blockIdx.x * kBlock + threadIdx.x;
    const unsigned long long at = slot - skew;
    const bool live_vec = slot >= skew && at < nvec;
    uint4 v = uint4{0u, 0u, 0u, 0u};
    if (live_vec) {
        if constexpr (IN_UNALIGNED) v = load_stream_unaligned(reinterpret_cast<const char *>(vin) + 16 * at);
        else v = load_stream(vin + at);
    }
    const uint2 o = narrow_ktanh_vec(v, tab);
    if (live_vec) store_stream(vout + at, o);

    if (n_edge != 0 && blockIdx.x == 0) {  // uniform over the block
        const unsigned k = threadIdx.x;
        const bool live = k < n_edge;
        const unsigned long long i = k < edge.n_head ? k : edge.n_total - n_edge + k;
        uint32_t x = 0;
        if (live) x = static_cast<const uint32_t *>(edge.ein)[i];
        x = ktanh_pair(narrow_pair(__uint_as_float(x), 0.0f), tab);
        if (live) static_cast<uint16_t *>(edge.eout)[i] = (uint16_t)x;
    }
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
    const unsigned n_edge = (unsigned)(head + tail);
    const unsigned skew = (unsigned)((reinterpret_cast<uintptr_t>(out + head) / 8) % kBlock);
    size_t tiles = (nvec + skew + kBlock - 1) / kBlock;
    if (tiles == 0) tiles = 1;
    if (tiles > kMaxTiles) return KT_ERR_SHAPE;
    const uint4 *vin = reinterpret_cast<const uint4 *>(in + head);
    uint2 *vout = reinterpret_cast<uint2 *>(out + head);
    if (reinterpret_cast<uintptr_t>(vin) % 16 == 0)
        return launch_checked(narrow_stream_kernel<false>, (unsigned)tiles, kBlock, stream, vin, vout,
                              (unsigned long long)nvec, skew, n_edge, edge, pack);
    return launch_checked(narrow_stream_kernel<true>, (unsigned)tiles, kBlock, stream, vin, vout,
                          (unsigned long long)nvec, skew, n_edge, edge, pack);
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

extern "C" ktanh_status_t kpade32_bf16(const uint16_t *in, uint16_t *out, size_t n, ktanh_stream_t stream)
{
    return launch_elementwise<false, OP_PADE32>(in, out, n, static_cast<const ktanh_lut_t *>(nullptr), stream);
}

extern "C" ktanh_status_t kpade78_bf16(const uint16_t *in, uint16_t *out, size_t n, ktanh_stream_t stream)
{
    return launch_elementwise<false, OP_PADE78>(in, out, n, static_cast<const ktanh_lut_t *>(nullptr), stream);
}

extern "C" ktanh_status_t ktaylor2_bf16(const uint16_t *in, uint16_t *out, size_t n, ktanh_stream_t stream)
{
    return launch_elementwise<false, OP_TAYLOR2>(in, out, n, static_cast<const ktanh_lut_t *>(nullptr), stream);
}

extern "C" ktanh_status_t ktaylor3_bf16(const uint16_t *in, uint16_t *out, size_t n, ktanh_stream_t stream)
{
    return launch_elementwise<false, OP_TAYLOR3>(in, out, n, static_cast<const ktanh_lut_t *>(nullptr), stream);
}
