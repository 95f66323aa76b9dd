// libktanh: gradients for training through K-TanH -- the derivative identities of TanH and Sigmoid
// on the forward outputs, the derivatives of the Swish and GELU identities from the forward inputs
// (BFloat16 and Float32 tensors), and one LSTM-cell step backwards -- and their entry points.
#include "ktanh_device.h"

using namespace ktanh_device;

namespace {

// Which slope multiplies dy.  TanH and Sigmoid take it from the forward OUTPUT (no table involved);
// Swish and GELU rebuild the K-TanH value from the forward INPUT with the device functions the
// forward kernels use:
//   TanH'    = 1 - y^2                      Sigmoid' = s * (1 - s)
//   Swish'   = s + x * (s * (1 - s)),                                       s = Sigmoid(x)
//   GELU'    = 0.5 * (1 + t) + (0.5 * x) * ((1 - t^2) * (c * (1 + 3a * x^2))),   t = K(c * (x + a x^3))
// Float32, one rounding per written operation.
enum Grad { GRAD_TANH = 0, GRAD_SIGMOID = 1, GRAD_SWISH = 2, GRAD_GELU = 3 };

// The slope from Float32 values: v is the forward output (TanH, Sigmoid) or the input with its
// K-TanH-derived value k already formed (s for Swish, t for GELU).
template <int GRAD>
__device__ __forceinline__ float slope_of(float v, float k)
{
    if constexpr (GRAD == GRAD_TANH) {
        const float sq = v * v;
        return 1.0f - sq;
    } else if constexpr (GRAD == GRAD_SIGMOID) {
        const float one_minus = 1.0f - v;
        return v * one_minus;
    } else if constexpr (GRAD == GRAD_SWISH) {
        const float one_minus = 1.0f - k;
        const float bell = k * one_minus;
        const float xbell = v * bell;
        return k + xbell;
    } else {
        const float a3 = 0.134145f;  // 3a
        const float c = 0.7978845608028654f;
        const float one_plus = 1.0f + k;
        const float left = 0.5f * one_plus;
        const float tsq = k * k;
        const float sech2 = 1.0f - tsq;
        const float sq = v * v;
        const float a3sq = a3 * sq;
        const float poly = 1.0f + a3sq;
        const float du = c * poly;
        const float chain = sech2 * du;
        const float half_x = 0.5f * v;
        const float right = half_x * chain;
        return left + right;
    }
}

// The argument of K inside GELU: c * (x + a * x^3).
__device__ __forceinline__ float gelu_argument(float x)
{
    const float a = 0.044715f;
    const float c = 0.7978845608028654f;
    const float sq = x * x;
    const float cube = sq * x;
    const float acube = a * cube;
    const float inner = x + acube;
    return c * inner;
}

// One 32-bit word of each stream: a packed BFloat16 pair (ELEM = uint16_t) or one Float32
// (ELEM = uint32_t).  A single BFloat16 element travels in the low half of the word.
template <class ELEM, int GRAD, bool WIDE>
__device__ __forceinline__ uint32_t grad_word(uint32_t dy_w, uint32_t v_w, const LaneTable &tab)
{
    if constexpr (sizeof(ELEM) == 2) {
        const float dy[2] = {widen_lo(dy_w), widen_hi(dy_w)};
        const float v[2] = {widen_lo(v_w), widen_hi(v_w)};
        float k[2] = {0.f, 0.f};
        if constexpr (GRAD == GRAD_SWISH) {
            ksigmoid_f32_pair<false, WIDE>(v_w, tab, k[0], k[1]);  // a NaN x reaches the slope through x itself
        } else if constexpr (GRAD == GRAD_GELU) {
            const uint32_t t2 = ktanh_pair<false, WIDE>(narrow_pair(gelu_argument(v[0]), gelu_argument(v[1])), tab);
            k[0] = widen_lo(t2);
            k[1] = widen_hi(t2);
        }
        return narrow_pair(dy[0] * slope_of<GRAD>(v[0], k[0]), dy[1] * slope_of<GRAD>(v[1], k[1]));
    } else {
        const float dy = __uint_as_float(dy_w), v = __uint_as_float(v_w);
        float k = 0.f;
        if constexpr (GRAD == GRAD_SWISH) {
            // 0.5 * t is exact for every K output t that can change the sum, so the multiply-add may fuse
            const float t = __uint_as_float(ktanh_f32_one<WIDE>(__float_as_uint(0.5f * v), tab));
            k = __builtin_fmaf(0.5f, t, 0.5f);
        } else if constexpr (GRAD == GRAD_GELU) {
            k = __uint_as_float(ktanh_f32_one<WIDE>(__float_as_uint(gelu_argument(v)), tab));
        }
        return __float_as_uint(dy * slope_of<GRAD>(v, k));
    }
}

// Two input streams, one output stream (which may be one of the inputs): 6 bytes per BFloat16
// element, 12 per Float32 element.  One wavefront per block, one 128-bit vector per lane and stream.
// The body starts where `dx` reaches a 16-byte boundary and its tiles are cut at 1 KiB boundaries of
// `dx` (skew = index of the first vector inside its 1 KiB group); the elements before and after the
// body (n_edge < 64 of them) are taken by block 0.  IN_UNALIGNED: an input disagrees with `dx`
// modulo 16 bytes, so both are read with 16-byte loads from element-aligned addresses.  The table
// reads of Swish and GELU need every lane enabled, so bounds predicate only the loads and stores.
// The arguments a wavefront needs before its loads (the three body pointers, nvec, skew, n_edge)
// come first, as scalars: the leading scalar arguments of a kernel arrive preloaded in registers.
template <class ELEM>
struct GradEdge {
    const ELEM *dy, *v;  // the whole tensors
    ELEM *dx;
    unsigned long long n;
    unsigned n_head;
};

template <class ELEM, int GRAD, bool WIDE, bool IN_UNALIGNED>
__global__ __launch_bounds__(kBlock) void grad_stream_kernel(const char *bdy0, const char *bv0,
                                                             uint4 *bdx0,  // the aligned bodies
                                                             unsigned long long nvec, unsigned skew,
                                                             unsigned n_edge, unsigned whole,
                                                             unsigned lg_seg,  // TileOrder
                                                             GradEdge<ELEM> g, KtLutPack pack)
{
    const LaneTable tab(pack);
    const unsigned long long slot =
        (unsigned long long)tile_of_block(blockIdx.x, whole, lg_seg) * kBlock + threadIdx.x;
    const unsigned long long at = slot - skew;
    const bool live = slot >= skew && at < nvec;
    const char *bdy = bdy0 + 16 * at;
    const char *bv = bv0 + 16 * at;
    uint4 a = uint4{0u, 0u, 0u, 0u}, b = uint4{0u, 0u, 0u, 0u};
    if (live) {
        if constexpr (IN_UNALIGNED) {
            a = load_stream_unaligned(bdy);
            b = load_stream_unaligned(bv);
        } else {
            a = load_stream(reinterpret_cast<const uint4 *>(bdy));
            b = load_stream(reinterpret_cast<const uint4 *>(bv));
        }
    }
    const uint4 r = uint4{grad_word<ELEM, GRAD, WIDE>(a.x, b.x, tab), grad_word<ELEM, GRAD, WIDE>(a.y, b.y, tab),
                          grad_word<ELEM, GRAD, WIDE>(a.z, b.z, tab), grad_word<ELEM, GRAD, WIDE>(a.w, b.w, tab)};
    if (live) store_stream(bdx0 + at, r);
    if (n_edge != 0 && blockIdx.x == 0) {  // uniform over the block
        const unsigned k = threadIdx.x;
        const bool some = k < n_edge;
        const unsigned long long i = k < g.n_head ? k : g.n - n_edge + k;
        const uint32_t d1 = some ? g.dy[i] : 0u, v1 = some ? g.v[i] : 0u;
        const uint32_t r1 = grad_word<ELEM, GRAD, WIDE>(d1, v1, tab);
        if (some) g.dx[i] = (ELEM)r1;
    }
}

ktanh_status_t pack_grad(const ktanh_lut_t *lut, bool f32, KtLutPack *pack)
{
    return f32 ? kt_pack_lut_f32(lut, pack) : kt_pack_lut_bf16(lut, pack);
}
ktanh_status_t pack_grad(const ktanh_lut64_t *lut, bool f32, KtLutPack *pack)
{
    return f32 ? kt_pack_lut64_f32(lut, pack) : kt_pack_lut64_bf16(lut, pack);
}
// `lut` is only read by Swish and GELU; TanH and Sigmoid pass NULL and Table 1 rides along unused.
template <class ELEM, int GRAD, class Lut>
ktanh_status_t launch_grad(const void *dy, const void *v, void *dx, size_t n, const Lut *lut,
                           ktanh_stream_t stream)
{
    constexpr bool WIDE = is_wide(static_cast<const Lut *>(nullptr));
    constexpr size_t kPerVec = 16 / sizeof(ELEM);
    if (n == 0) return KT_OK;
    if (dy == nullptr || v == nullptr || dx == nullptr) return KT_ERR_NULL;
    const uintptr_t ady = reinterpret_cast<uintptr_t>(dy), av = reinterpret_cast<uintptr_t>(v),
                    adx = reinterpret_cast<uintptr_t>(dx);
    if ((ady | av | adx) & (sizeof(ELEM) - 1)) return KT_ERR_ALIGN;
    if (n > (size_t)1 << 40) return KT_ERR_SHAPE;
    KtLutPack pack;
    const ktanh_status_t st = pack_grad(lut, sizeof(ELEM) == 4, &pack);
    if (st != KT_OK) return st;
    GradEdge<ELEM> g;
    g.dy = static_cast<const ELEM *>(dy);
    g.v = static_cast<const ELEM *>(v);
    g.dx = static_cast<ELEM *>(dx);
    g.n = n;
    size_t head = ((16 - (adx & 15)) & 15) / sizeof(ELEM);
    if (head > n) head = n;
    const size_t nvec = (n - head) / kPerVec;
    g.n_head = (unsigned)head;
    const unsigned n_edge = (unsigned)(n - nvec * kPerVec);
    const unsigned skew = (unsigned)((reinterpret_cast<uintptr_t>(g.dx + head) / 16) % kBlock);
    size_t tiles = (nvec + skew + kBlock - 1) / kBlock;
    if (tiles == 0) tiles = 1;  // edge elements only
    if (tiles > kMaxTiles) return KT_ERR_SHAPE;
    const char *bdy = reinterpret_cast<const char *>(g.dy + head);
    const char *bv = reinterpret_cast<const char *>(g.v + head);
    uint4 *bdx = reinterpret_cast<uint4 *>(g.dx + head);
    // three streams: the two-window order of the forward kernels measured 1.3 % slower here
    const TileOrder order = TileOrder{0u, 18u};
    if ((ady & 15) == (adx & 15) && (av & 15) == (adx & 15))
        return launch_checked(grad_stream_kernel<ELEM, GRAD, WIDE, false>, (unsigned)tiles, kBlock, stream,
                              bdy, bv, bdx, (unsigned long long)nvec, skew, n_edge, order.whole,
                              order.lg_seg, g, pack);
    return launch_checked(grad_stream_kernel<ELEM, GRAD, WIDE, true>, (unsigned)tiles, kBlock, stream, bdy,
                          bv, bdx, (unsigned long long)nvec, skew, n_edge, order.whole, order.lg_seg, g,
                          pack);
}

// ---------------------------------------------------------------------------------------------
// LSTM cell, one step backwards: each lane owns two neighbouring cells (one packed pair per gate).
// The forward activations are rebuilt with the same device functions the forward kernel uses; the
// table reads need every lane enabled, so bounds predicate only the memory accesses.
constexpr int kCellBlock = 256;

template <bool WIDE>
__global__ __launch_bounds__(kCellBlock) void lstm_cell_backward_kernel(
    const uint32_t *__restrict__ gates, const float2 *__restrict__ c_prev,
    const uint32_t *__restrict__ dh, const float2 *dc_next, uint32_t *__restrict__ dgates,
    float2 *dc_prev, unsigned n_pairs, unsigned H2, KtLutPack pack)
{
    const LaneTable tab(pack);
    const unsigned p = blockIdx.x * kCellBlock + threadIdx.x;
    const bool live = p < n_pairs;
    const unsigned b = live ? p / H2 : 0;
    const unsigned j = live ? p % H2 : 0;
    const unsigned at = b * 4u * H2 + j;  // word index of the i-gate pair inside [B][4H]

    uint32_t wi = 0, wf = 0, wg = 0, wo = 0, wdh = 0;
    float2 c0 = float2{0.f, 0.f}, dcn = float2{0.f, 0.f};
    if (live) {
        wi = gates[at];
        wf = gates[at + H2];
        wg = gates[at + 2u * H2];
        wo = gates[at + 3u * H2];
        wdh = dh[p];
        c0 = c_prev[p];
        dcn = dc_next[p];
    }

    float ig[2], fg[2], og[2];
    ksigmoid_f32_pair<true, WIDE>(wi, tab, ig[0], ig[1]);
    ksigmoid_f32_pair<true, WIDE>(wf, tab, fg[0], fg[1]);
    ksigmoid_f32_pair<true, WIDE>(wo, tab, og[0], og[1]);
    const uint32_t g2 = ktanh_pair<true, WIDE>(wg, tab);
    const float gg[2] = {widen_lo(g2), widen_hi(g2)};
    const float cp[2] = {c0.x, c0.y};
    float c1[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const float keep = fg[k] * cp[k], add = ig[k] * gg[k];
        c1[k] = keep + add;
    }
    const uint32_t tc2 = ktanh_pair<true, WIDE>(narrow_pair(c1[0], c1[1]), tab);
    const float tc[2] = {widen_lo(tc2), widen_hi(tc2)};
    const float dhv[2] = {widen_lo(wdh), widen_hi(wdh)};
    const float dnx[2] = {dcn.x, dcn.y};

    float d_gi[2], d_gf[2], d_gg[2], d_go[2], dcp[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const float d_o = dhv[k] * tc[k];
        const float dh_o = dhv[k] * og[k];
        const float tsq = tc[k] * tc[k];
        const float tslope = 1.0f - tsq;
        const float through = dh_o * tslope;
        const float dc = dnx[k] + through;
        const float d_i = dc * gg[k], d_f = dc * cp[k], d_g = dc * ig[k];
        dcp[k] = dc * fg[k];
        const float i1 = 1.0f - ig[k], f1 = 1.0f - fg[k], o1 = 1.0f - og[k];
        const float islope = ig[k] * i1, fslope = fg[k] * f1, oslope = og[k] * o1;
        const float gsq = gg[k] * gg[k];
        const float gslope = 1.0f - gsq;
        d_gi[k] = d_i * islope;
        d_gf[k] = d_f * fslope;
        d_gg[k] = d_g * gslope;
        d_go[k] = d_o * oslope;
    }
    if (live) {
        dgates[at] = narrow_pair(d_gi[0], d_gi[1]);
        dgates[at + H2] = narrow_pair(d_gf[0], d_gf[1]);
        dgates[at + 2u * H2] = narrow_pair(d_gg[0], d_gg[1]);
        dgates[at + 3u * H2] = narrow_pair(d_go[0], d_go[1]);
        dc_prev[p] = float2{dcp[0], dcp[1]};
    }
}

}  // namespace

extern "C" ktanh_status_t ktanh_bf16_backward(const uint16_t *dy, const uint16_t *y, uint16_t *dx,
                                              size_t n, ktanh_stream_t stream)
{
    return launch_grad<uint16_t, GRAD_TANH>(dy, y, dx, n, static_cast<const ktanh_lut_t *>(nullptr), stream);
}

extern "C" ktanh_status_t ksigmoid_backward(const uint16_t *dy, const uint16_t *s, uint16_t *dx,
                                            size_t n, ktanh_stream_t stream)
{
    return launch_grad<uint16_t, GRAD_SIGMOID>(dy, s, dx, n, static_cast<const ktanh_lut_t *>(nullptr), stream);
}

extern "C" ktanh_status_t kswish_backward(const uint16_t *dy, const uint16_t *x, uint16_t *dx,
                                          size_t n, const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    return launch_grad<uint16_t, GRAD_SWISH>(dy, x, dx, n, lut, stream);
}

extern "C" ktanh_status_t kgelu_backward(const uint16_t *dy, const uint16_t *x, uint16_t *dx,
                                         size_t n, const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    return launch_grad<uint16_t, GRAD_GELU>(dy, x, dx, n, lut, stream);
}

extern "C" ktanh_status_t ktanh_f32_backward(const float *dy, const float *y, float *dx, size_t n,
                                             ktanh_stream_t stream)
{
    return launch_grad<uint32_t, GRAD_TANH>(dy, y, dx, n, static_cast<const ktanh_lut_t *>(nullptr), stream);
}

extern "C" ktanh_status_t ksigmoid_f32_backward(const float *dy, const float *s, float *dx, size_t n,
                                                ktanh_stream_t stream)
{
    return launch_grad<uint32_t, GRAD_SIGMOID>(dy, s, dx, n, static_cast<const ktanh_lut_t *>(nullptr), stream);
}

extern "C" ktanh_status_t kswish_f32_backward(const float *dy, const float *x, float *dx, size_t n,
                                              const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    return launch_grad<uint32_t, GRAD_SWISH>(dy, x, dx, n, lut, stream);
}

extern "C" ktanh_status_t kgelu_f32_backward(const float *dy, const float *x, float *dx, size_t n,
                                             const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    return launch_grad<uint32_t, GRAD_GELU>(dy, x, dx, n, lut, stream);
}

namespace {

ktanh_status_t pack_cell(const ktanh_lut_t *lut, KtLutPack *pack) { return kt_pack_lut_bf16(lut, pack); }
ktanh_status_t pack_cell(const ktanh_lut64_t *lut, KtLutPack *pack) { return kt_pack_lut64_bf16(lut, pack); }

template <class Lut>
ktanh_status_t launch_cell_backward(const uint16_t *gates, const float *c_prev, const uint16_t *dh,
                                    const float *dc_next, uint16_t *dgates, float *dc_prev, size_t B,
                                    size_t H, const Lut *lut, ktanh_stream_t stream)
{
    constexpr bool WIDE = is_wide(static_cast<const Lut *>(nullptr));
    if (B == 0 || H == 0) return KT_OK;
    if (gates == nullptr || c_prev == nullptr || dh == nullptr || dc_next == nullptr ||
        dgates == nullptr || dc_prev == nullptr)
        return KT_ERR_NULL;
    if (H % 8 != 0) return KT_ERR_SHAPE;
    if (B > ((size_t)1 << 40) || H > ((size_t)1 << 40)) return KT_ERR_SHAPE;
    // the kernel moves BFloat16 pairs (4 bytes) and Float32 pairs (8 bytes)
    const uintptr_t words = reinterpret_cast<uintptr_t>(gates) | reinterpret_cast<uintptr_t>(dh) |
                            reinterpret_cast<uintptr_t>(dgates);
    const uintptr_t states = reinterpret_cast<uintptr_t>(c_prev) | reinterpret_cast<uintptr_t>(dc_next) |
                             reinterpret_cast<uintptr_t>(dc_prev);
    if ((words & 3) || (states & 7)) return KT_ERR_ALIGN;
    KtLutPack pack;
    const ktanh_status_t st = pack_cell(lut, &pack);
    if (st != KT_OK) return st;
    if (B > (1ull << 28) / (H / 2)) return KT_ERR_SHAPE;
    const unsigned long long n_pairs = (unsigned long long)B * (H / 2);
    if (n_pairs >= (1ull << 28)) return KT_ERR_SHAPE;  // word indices inside [B][4H] fit 32 bits
    const unsigned long long blocks = (n_pairs + kCellBlock - 1) / kCellBlock;
    return launch_checked(lstm_cell_backward_kernel<WIDE>, (unsigned)blocks, kCellBlock, stream,
                          reinterpret_cast<const uint32_t *>(gates),
                          reinterpret_cast<const float2 *>(c_prev),
                          reinterpret_cast<const uint32_t *>(dh),
                          reinterpret_cast<const float2 *>(dc_next),
                          reinterpret_cast<uint32_t *>(dgates), reinterpret_cast<float2 *>(dc_prev),
                          (unsigned)n_pairs, (unsigned)(H / 2), pack);
}

}  // namespace

extern "C" ktanh_status_t klstm_cell_backward(const uint16_t *gates, const float *c_prev,
                                              const uint16_t *dh, const float *dc_next,
                                              uint16_t *dgates, float *dc_prev, size_t B, size_t H,
                                              const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    return launch_cell_backward(gates, c_prev, dh, dc_next, dgates, dc_prev, B, H, lut, stream);
}

extern "C" ktanh_status_t klstm_cell64_backward(const uint16_t *gates, const float *c_prev,
                                                const uint16_t *dh, const float *dc_next,
                                                uint16_t *dgates, float *dc_prev, size_t B, size_t H,
                                                const ktanh_lut64_t *lut, ktanh_stream_t stream)
{
    return launch_cell_backward(gates, c_prev, dh, dc_next, dgates, dc_prev, B, H, lut, stream);
}

extern "C" ktanh_status_t kswish64_backward(const uint16_t *dy, const uint16_t *x, uint16_t *dx,
                                            size_t n, const ktanh_lut64_t *lut, ktanh_stream_t stream)
{
    return launch_grad<uint16_t, GRAD_SWISH>(dy, x, dx, n, lut, stream);
}

extern "C" ktanh_status_t kgelu64_backward(const uint16_t *dy, const uint16_t *x, uint16_t *dx,
                                           size_t n, const ktanh_lut64_t *lut, ktanh_stream_t stream)
{
    return launch_grad<uint16_t, GRAD_GELU>(dy, x, dx, n, lut, stream);
}

extern "C" ktanh_status_t kswish64_f32_backward(const float *dy, const float *x, float *dx, size_t n,
                                                const ktanh_lut64_t *lut, ktanh_stream_t stream)
{
    return launch_grad<uint32_t, GRAD_SWISH>(dy, x, dx, n, lut, stream);
}

extern "C" ktanh_status_t kgelu64_f32_backward(const float *dy, const float *x, float *dx, size_t n,
                                               const ktanh_lut64_t *lut, ktanh_stream_t stream)
{
    return launch_grad<uint32_t, GRAD_GELU>(dy, x, dx, n, lut, stream);
}
