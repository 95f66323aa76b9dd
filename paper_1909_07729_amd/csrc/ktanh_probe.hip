// libktanh_probe: measurement yardsticks, not operations of the paper.  Each is the launch of the
// element-wise entry points (one wavefront per block, one 128-bit vector per lane, the same load and
// store policies) with the arithmetic, the stores or the loads taken out, so that a benchmark can
// put what the memory system allows for this launch shape next to the K-TanH figures.  Likewise the
// launch of the fused LSTM-cell kernel with its arithmetic taken out.
#include "ktanh_probe.h"
#include "ktanh_lstm_impl.h"
#include "ktanh_stream_impl.h"

using namespace ktanh_device;

namespace {

constexpr int kWide = 512;  // eight wavefronts per block

// Loads only: the store is kept in the code behind a test no benchmark tensor passes, so that the
// loads stay; if it ever fires it writes inside `sink` (1 KiB, one vector per lane).
// THREADS = 64 is the library's launch shape; 512 (eight wavefronts per block) asks the dispatcher for
// an eighth of the blocks and shows what the memory system gives to loads alone.
template <int THREADS>
__global__ __launch_bounds__(THREADS) void read_kernel(const uint4 *__restrict__ vin, uint4 *sink,
                                                       unsigned long long nvec)
{
    const unsigned long long at = (unsigned long long)blockIdx.x * THREADS + threadIdx.x;
    if (at >= nvec) return;
    const uint4 v = load_stream(vin + at);
    if ((v.x ^ v.y) == 0x7FC1A5A5u && (v.z ^ v.w) == 0x5A5A1CF7u) store_stream(sink + (threadIdx.x & 63), v);
}

// Stores only: a fixed pattern.
template <int THREADS>
__global__ __launch_bounds__(THREADS) void write_kernel(uint4 *__restrict__ vout, unsigned long long nvec)
{
    const unsigned long long at = (unsigned long long)blockIdx.x * THREADS + threadIdx.x;
    if (at >= nvec) return;
    store_stream(vout + at, uint4{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u});
}

ktanh_status_t check(const void *p, size_t n_bytes, unsigned long long *tiles)
{
    if (p == nullptr) return KT_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(p) % 1024 != 0) return KT_ERR_ALIGN;
    if (n_bytes % 16 != 0) return KT_ERR_SHAPE;
    *tiles = (n_bytes / 16 + kBlock - 1) / kBlock;
    return *tiles > kMaxTiles ? KT_ERR_SHAPE : KT_OK;
}

}  // namespace

extern "C" ktanh_status_t ktanh_probe_copy(const uint16_t *in, uint16_t *out, size_t n,
                                           ktanh_stream_t stream)
{
    return launch_elementwise<false, OP_COPY>(in, out, n, static_cast<const ktanh_lut_t *>(nullptr), stream);
}

extern "C" ktanh_status_t ktanh_probe_read(const void *in, void *sink, size_t n_bytes,
                                           ktanh_stream_t stream)
{
    if (n_bytes == 0) return KT_OK;
    unsigned long long tiles = 0;
    const ktanh_status_t st = check(in, n_bytes, &tiles);
    if (st != KT_OK) return st;
    if (sink == nullptr) return KT_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(sink) % 16 != 0) return KT_ERR_ALIGN;
    return launch_checked(read_kernel<kBlock>, (unsigned)tiles, kBlock, stream, static_cast<const uint4 *>(in),
                          static_cast<uint4 *>(sink), (unsigned long long)(n_bytes / 16));
}

extern "C" ktanh_status_t ktanh_probe_read_wide(const void *in, void *sink, size_t n_bytes,
                                                ktanh_stream_t stream)
{
    if (n_bytes == 0) return KT_OK;
    unsigned long long tiles = 0;
    const ktanh_status_t st = check(in, n_bytes, &tiles);
    if (st != KT_OK) return st;
    if (sink == nullptr) return KT_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(sink) % 16 != 0) return KT_ERR_ALIGN;
    return launch_checked(read_kernel<kWide>, (unsigned)((tiles + 7) / 8), kWide, stream,
                          static_cast<const uint4 *>(in), static_cast<uint4 *>(sink),
                          (unsigned long long)(n_bytes / 16));
}

extern "C" ktanh_status_t ktanh_probe_write(void *out, size_t n_bytes, ktanh_stream_t stream)
{
    if (n_bytes == 0) return KT_OK;
    unsigned long long tiles = 0;
    const ktanh_status_t st = check(out, n_bytes, &tiles);
    if (st != KT_OK) return st;
    return launch_checked(write_kernel<kBlock>, (unsigned)tiles, kBlock, stream, static_cast<uint4 *>(out),
                          (unsigned long long)(n_bytes / 16));
}

extern "C" ktanh_status_t ktanh_probe_write_wide(void *out, size_t n_bytes, ktanh_stream_t stream)
{
    if (n_bytes == 0) return KT_OK;
    unsigned long long tiles = 0;
    const ktanh_status_t st = check(out, n_bytes, &tiles);
    if (st != KT_OK) return st;
    return launch_checked(write_kernel<kWide>, (unsigned)((tiles + 7) / 8), kWide, stream,
                          static_cast<uint4 *>(out), (unsigned long long)(n_bytes / 16));
}

extern "C" ktanh_status_t ktanh_probe_lstm(const uint16_t *gates, const float *c_in, float *c_out,
                                           uint16_t *h_out, size_t T, size_t B, size_t H,
                                           ktanh_stream_t stream)
{
    return launch_cell<false, false>(gates, c_in, c_out, h_out, T, B, H,
                                     static_cast<const ktanh_lut_t *>(nullptr), stream);
}
