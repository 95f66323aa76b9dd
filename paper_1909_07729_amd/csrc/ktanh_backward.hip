// libktanh: gradients for training through K-TanH -- the derivative identities of TanH and Sigmoid
// on the forward outputs, the derivatives of the Swish and GELU identities from the forward inputs,
// and one LSTM-cell step backwards -- and their entry points.
#include "ktanh_device.h"

using namespace ktanh_device;

namespace {

enum Grad { GRAD_TANH = 0, GRAD_SIGMOID = 1 };

// dy * slope(forward output) for both halves of a packed pair.
template <int GRAD>
__device__ __forceinline__ uint32_t grad_pair(uint32_t dy2, uint32_t fwd2)
{
    float out[2];
    const float dy[2] = {widen_lo(dy2), widen_hi(dy2)};
    const float v[2] = {widen_lo(fwd2), widen_hi(fwd2)};
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        float slope;
        if constexpr (GRAD == GRAD_TANH) {
            const float sq = v[k] * v[k];
            slope = 1.0f - sq;
        } else {
            const float one_minus = 1.0f - v[k];
            slope = v[k] * one_minus;
        }
        out[k] = dy[k] * slope;
    }
    return narrow_pair(out[0], out[1]);
}

// Two BFloat16 input streams, one output stream (which may be one of the inputs): 6 bytes per element.  One wavefront per block,
// one 128-bit vector per lane; the last block also takes the n % 8 loose elements.
template <int GRAD>
__global__ __launch_bounds__(kBlock) void grad_stream_kernel(const uint4 *vdy,
                                                             const uint4 *vfwd,
                                                             uint4 *vdx,
                                                             unsigned long long nvec,
                                                             const uint16_t *dy, const uint16_t *fwd,
                                                             uint16_t *dx, unsigned long long n)
{
    const unsigned long long at = (unsigned long long)blockIdx.x * kBlock + threadIdx.x;
    if (at < nvec) {
        const uint4 a = load_stream(vdy + at), b = load_stream(vfwd + at);
        store_stream(vdx + at, uint4{grad_pair<GRAD>(a.x, b.x), grad_pair<GRAD>(a.y, b.y),
                                     grad_pair<GRAD>(a.z, b.z), grad_pair<GRAD>(a.w, b.w)});
    }
    const unsigned long long loose = nvec * 8 + threadIdx.x;
    if (blockIdx.x == gridDim.x - 1 && loose < n) dx[loose] = (uint16_t)grad_pair<GRAD>(dy[loose], fwd[loose]);
}

// Any alignment: one element per lane and pass.
template <int GRAD>
__global__ __launch_bounds__(kBlock) void grad_element_kernel(const uint16_t *dy,
                                                              const uint16_t *fwd,
                                                              uint16_t *dx,
                                                              unsigned long long n)
{
    const unsigned long long stride = (unsigned long long)gridDim.x * kBlock;
    for (unsigned long long i = (unsigned long long)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride)
        dx[i] = (uint16_t)grad_pair<GRAD>(dy[i], fwd[i]);
}

template <int GRAD>
ktanh_status_t launch_grad(const uint16_t *dy, const uint16_t *fwd, uint16_t *dx, size_t n,
                           ktanh_stream_t stream)
{
    if (n == 0) return KT_OK;
    if (dy == nullptr || fwd == nullptr || dx == nullptr) return KT_ERR_NULL;
    const uintptr_t all = reinterpret_cast<uintptr_t>(dy) | reinterpret_cast<uintptr_t>(fwd) |
                          reinterpret_cast<uintptr_t>(dx);
    if (all & 1) return KT_ERR_ALIGN;
    if (n > (size_t)1 << 40) return KT_ERR_SHAPE;
    if ((all & 15) == 0) {
        const size_t nvec = n / 8;
        size_t tiles = (nvec + kBlock - 1) / kBlock;
        if (tiles == 0) tiles = 1;
        if (tiles > 0x7FFFFFFFull) return KT_ERR_SHAPE;
        return launch_checked(grad_stream_kernel<GRAD>, (unsigned)tiles, kBlock, stream,
                              reinterpret_cast<const uint4 *>(dy), reinterpret_cast<const uint4 *>(fwd),
                              reinterpret_cast<uint4 *>(dx), (unsigned long long)nvec, dy, fwd, dx,
                              (unsigned long long)n);
    }
    const size_t want = (n + kBlock - 1) / kBlock;
    return launch_checked(grad_element_kernel<GRAD>, (unsigned)(want < 8192 ? want : 8192), kBlock,
                          stream, dy, fwd, dx, (unsigned long long)n);
}

// ---------------------------------------------------------------------------------------------
// Swish and GELU: the slope needs the K-TanH value, which is rebuilt from the forward input x with
// the device functions the forward kernels use.
//   Swish' = s + x * (s * (1 - s)),                 s = Sigmoid(x)
//   GELU'  = 0.5 * (1 + t) + (0.5 * x) * ((1 - t^2) * (c * (1 + 3a * x^2))),   t = K(c * (x + a x^3))
// Float32, one rounding per written operation.
enum GradFromInput { GRAD_SWISH = 0, GRAD_GELU = 1 };

template <int GRAD>
__device__ __forceinline__ uint32_t grad_from_input_pair(uint32_t dy2, uint32_t x2,
                                                         const LaneTable &tab)
{
    const float dy[2] = {widen_lo(dy2), widen_hi(dy2)};
    const float x[2] = {widen_lo(x2), widen_hi(x2)};
    float slope[2];
    if constexpr (GRAD == GRAD_SWISH) {
        float s[2];
        ksigmoid_f32_pair<true, false>(x2, tab, s[0], s[1]);
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const float one_minus = 1.0f - s[k];
            const float bell = s[k] * one_minus;
            const float xbell = x[k] * bell;
            slope[k] = s[k] + xbell;
        }
    } else {
        const float a = 0.044715f;
        const float a3 = 0.134145f;
        const float c = 0.7978845608028654f;
        float sq[2], u[2];
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            sq[k] = x[k] * x[k];
            const float cube = sq[k] * x[k];
            const float acube = a * cube;
            const float inner = x[k] + acube;
            u[k] = c * inner;
        }
        const uint32_t t2 = ktanh_pair<true, false>(narrow_pair(u[0], u[1]), tab);
        const float t[2] = {widen_lo(t2), widen_hi(t2)};
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const float one_plus = 1.0f + t[k];
            const float left = 0.5f * one_plus;
            const float tsq = t[k] * t[k];
            const float sech2 = 1.0f - tsq;
            const float a3sq = a3 * sq[k];
            const float poly = 1.0f + a3sq;
            const float du = c * poly;
            const float chain = sech2 * du;
            const float half_x = 0.5f * x[k];
            const float right = half_x * chain;
            slope[k] = left + right;
        }
    }
    return narrow_pair(dy[0] * slope[0], dy[1] * slope[1]);
}

// Same shape as grad_stream_kernel.  The table reads need every lane enabled, so the bounds
// predicate only the loads and stores; the loose elements are taken by the whole last block.
template <int GRAD>
__global__ __launch_bounds__(kBlock) void grad_input_stream_kernel(
    const uint4 *vdy, const uint4 *vx, uint4 *vdx, unsigned long long nvec, const uint16_t *dy,
    const uint16_t *x, uint16_t *dx, unsigned long long n, KtLutPack pack)
{
    const LaneTable tab(pack);
    const unsigned long long at = (unsigned long long)blockIdx.x * kBlock + threadIdx.x;
    const bool live = at < nvec;
    uint4 a = uint4{0u, 0u, 0u, 0u}, b = uint4{0u, 0u, 0u, 0u};
    if (live) {
        a = load_stream(vdy + at);
        b = load_stream(vx + at);
    }
    const uint4 r = uint4{grad_from_input_pair<GRAD>(a.x, b.x, tab), grad_from_input_pair<GRAD>(a.y, b.y, tab),
                          grad_from_input_pair<GRAD>(a.z, b.z, tab), grad_from_input_pair<GRAD>(a.w, b.w, tab)};
    if (live) store_stream(vdx + at, r);
    if (blockIdx.x == gridDim.x - 1) {  // uniform over the block
        const unsigned long long loose = nvec * 8 + threadIdx.x;
        const bool some = loose < n;
        const uint32_t d1 = some ? dy[loose] : 0u, x1 = some ? x[loose] : 0u;
        const uint32_t r1 = grad_from_input_pair<GRAD>(d1, x1, tab);
        if (some) dx[loose] = (uint16_t)r1;
    }
}

// Any alignment: one element per lane and pass; the trip count is the same for the whole block.
template <int GRAD>
__global__ __launch_bounds__(kBlock) void grad_input_element_kernel(const uint16_t *dy,
                                                                    const uint16_t *x, uint16_t *dx,
                                                                    unsigned long long n,
                                                                    KtLutPack pack)
{
    const LaneTable tab(pack);
    const unsigned long long stride = (unsigned long long)gridDim.x * kBlock;
    for (unsigned long long base = (unsigned long long)blockIdx.x * kBlock; base < n; base += stride) {
        const unsigned long long i = base + threadIdx.x;
        const bool some = i < n;
        const uint32_t d1 = some ? dy[i] : 0u, x1 = some ? x[i] : 0u;
        const uint32_t r1 = grad_from_input_pair<GRAD>(d1, x1, tab);
        if (some) dx[i] = (uint16_t)r1;
    }
}

template <int GRAD>
ktanh_status_t launch_grad_from_input(const uint16_t *dy, const uint16_t *x, uint16_t *dx, size_t n,
                                      const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    if (n == 0) return KT_OK;
    if (dy == nullptr || x == nullptr || dx == nullptr) return KT_ERR_NULL;
    const uintptr_t all = reinterpret_cast<uintptr_t>(dy) | reinterpret_cast<uintptr_t>(x) |
                          reinterpret_cast<uintptr_t>(dx);
    if (all & 1) return KT_ERR_ALIGN;
    if (n > (size_t)1 << 40) return KT_ERR_SHAPE;
    KtLutPack pack;
    const ktanh_status_t st = kt_pack_lut_bf16(lut, &pack);
    if (st != KT_OK) return st;
    if ((all & 15) == 0) {
        const size_t nvec = n / 8;
        size_t tiles = (nvec + kBlock - 1) / kBlock;
        if (tiles == 0) tiles = 1;
        if (tiles > 0x7FFFFFFFull) return KT_ERR_SHAPE;
        return launch_checked(grad_input_stream_kernel<GRAD>, (unsigned)tiles, kBlock, stream,
                              reinterpret_cast<const uint4 *>(dy), reinterpret_cast<const uint4 *>(x),
                              reinterpret_cast<uint4 *>(dx), (unsigned long long)nvec, dy, x, dx,
                              (unsigned long long)n, pack);
    }
    const size_t want = (n + kBlock - 1) / kBlock;
    return launch_checked(grad_input_element_kernel<GRAD>, (unsigned)(want < 8192 ? want : 8192),
                          kBlock, stream, dy, x, dx, (unsigned long long)n, pack);
}

// ---------------------------------------------------------------------------------------------
// The same four gradients on Float32 tensors (12 bytes per element, four elements per 128-bit access).
// `v` is the forward output for TanH and Sigmoid and the forward input for Swish and GELU, whose
// K-TanH value is rebuilt with the Float32 form of Algorithm 1.
enum GradF32 { GF_TANH = 0, GF_SIGMOID = 1, GF_SWISH = 2, GF_GELU = 3 };

template <int GRAD>
__device__ __forceinline__ uint32_t grad_f32_one(uint32_t dy_bits, uint32_t v_bits, const LaneTable &tab)
{
    const float dy = __uint_as_float(dy_bits), v = __uint_as_float(v_bits);
    float slope;
    if constexpr (GRAD == GF_TANH) {
        const float sq = v * v;
        slope = 1.0f - sq;
    } else if constexpr (GRAD == GF_SIGMOID) {
        const float one_minus = 1.0f - v;
        slope = v * one_minus;
    } else if constexpr (GRAD == GF_SWISH) {
        // 0.5 * t is exact for every K output t that can change the sum, so the multiply-add may fuse
        const float t = __uint_as_float(ktanh_f32_one(__float_as_uint(0.5f * v), tab));
        const float s = __builtin_fmaf(0.5f, t, 0.5f);
        const float one_minus = 1.0f - s;
        const float bell = s * one_minus;
        const float xbell = v * bell;
        slope = s + xbell;
    } else {
        const float a = 0.044715f;
        const float a3 = 0.134145f;
        const float c = 0.7978845608028654f;
        const float sq = v * v;
        const float cube = sq * v;
        const float acube = a * cube;
        const float inner = v + acube;
        const float t = __uint_as_float(ktanh_f32_one(__float_as_uint(c * inner), tab));
        const float one_plus = 1.0f + t;
        const float left = 0.5f * one_plus;
        const float tsq = t * t;
        const float sech2 = 1.0f - tsq;
        const float a3sq = a3 * sq;
        const float poly = 1.0f + a3sq;
        const float du = c * poly;
        const float chain = sech2 * du;
        const float half_x = 0.5f * v;
        const float right = half_x * chain;
        slope = left + right;
    }
    return __float_as_uint(dy * slope);
}

// One wavefront per block, one 128-bit vector per lane and stream; every lane stays enabled around
// the table reads; the last block also takes the n % 4 loose elements.
template <int GRAD>
__global__ __launch_bounds__(kBlock) void grad_f32_stream_kernel(
    const uint4 *vdy, const uint4 *vv, uint4 *vdx, unsigned long long nvec, const uint32_t *dy,
    const uint32_t *v, uint32_t *dx, unsigned long long n, KtLutPack pack)
{
    const LaneTable tab(pack);
    const unsigned long long at = (unsigned long long)blockIdx.x * kBlock + threadIdx.x;
    const bool live = at < nvec;
    uint4 a = uint4{0u, 0u, 0u, 0u}, b = uint4{0u, 0u, 0u, 0u};
    if (live) {
        a = load_stream(vdy + at);
        b = load_stream(vv + at);
    }
    const uint4 r = uint4{grad_f32_one<GRAD>(a.x, b.x, tab), grad_f32_one<GRAD>(a.y, b.y, tab),
                          grad_f32_one<GRAD>(a.z, b.z, tab), grad_f32_one<GRAD>(a.w, b.w, tab)};
    if (live) store_stream(vdx + at, r);
    if (blockIdx.x == gridDim.x - 1) {  // uniform over the block
        const unsigned long long loose = nvec * 4 + threadIdx.x;
        const bool some = loose < n;
        const uint32_t d1 = some ? dy[loose] : 0u, v1 = some ? v[loose] : 0u;
        const uint32_t r1 = grad_f32_one<GRAD>(d1, v1, tab);
        if (some) dx[loose] = r1;
    }
}

template <int GRAD>
__global__ __launch_bounds__(kBlock) void grad_f32_element_kernel(const uint32_t *dy,
                                                                  const uint32_t *v, uint32_t *dx,
                                                                  unsigned long long n,
                                                                  KtLutPack pack)
{
    const LaneTable tab(pack);
    const unsigned long long stride = (unsigned long long)gridDim.x * kBlock;
    for (unsigned long long base = (unsigned long long)blockIdx.x * kBlock; base < n; base += stride) {
        const unsigned long long i = base + threadIdx.x;
        const bool some = i < n;
        const uint32_t d1 = some ? dy[i] : 0u, v1 = some ? v[i] : 0u;
        const uint32_t r1 = grad_f32_one<GRAD>(d1, v1, tab);
        if (some) dx[i] = r1;
    }
}

template <int GRAD>
ktanh_status_t launch_grad_f32(const float *dy, const float *v, float *dx, size_t n,
                               const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    if (n == 0) return KT_OK;
    if (dy == nullptr || v == nullptr || dx == nullptr) return KT_ERR_NULL;
    const uintptr_t all = reinterpret_cast<uintptr_t>(dy) | reinterpret_cast<uintptr_t>(v) |
                          reinterpret_cast<uintptr_t>(dx);
    if (all & 3) return KT_ERR_ALIGN;
    if (n > (size_t)1 << 40) return KT_ERR_SHAPE;
    KtLutPack pack;  // TanH and Sigmoid need no table: Table 1 rides along unused
    const ktanh_status_t st = kt_pack_lut_f32(lut, &pack);
    if (st != KT_OK) return st;
    const uint32_t *udy = reinterpret_cast<const uint32_t *>(dy), *uv = reinterpret_cast<const uint32_t *>(v);
    uint32_t *udx = reinterpret_cast<uint32_t *>(dx);
    if ((all & 15) == 0) {
        const size_t nvec = n / 4;
        size_t tiles = (nvec + kBlock - 1) / kBlock;
        if (tiles == 0) tiles = 1;
        if (tiles > 0x7FFFFFFFull) return KT_ERR_SHAPE;
        return launch_checked(grad_f32_stream_kernel<GRAD>, (unsigned)tiles, kBlock, stream,
                              reinterpret_cast<const uint4 *>(dy), reinterpret_cast<const uint4 *>(v),
                              reinterpret_cast<uint4 *>(dx), (unsigned long long)nvec, udy, uv, udx,
                              (unsigned long long)n, pack);
    }
    const size_t want = (n + kBlock - 1) / kBlock;
    return launch_checked(grad_f32_element_kernel<GRAD>, (unsigned)(want < 8192 ? want : 8192),
                          kBlock, stream, udy, uv, udx, (unsigned long long)n, pack);
}

// ---------------------------------------------------------------------------------------------
// LSTM cell, one step backwards: each lane owns two neighbouring cells (one packed pair per gate).
// The forward activations are rebuilt with the same device functions the forward kernel uses; the
// table reads need every lane enabled, so bounds predicate only the memory accesses.
constexpr int kCellBlock = 256;

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
    ksigmoid_f32_pair(wi, tab, ig[0], ig[1]);
    ksigmoid_f32_pair(wf, tab, fg[0], fg[1]);
    ksigmoid_f32_pair(wo, tab, og[0], og[1]);
    const uint32_t g2 = ktanh_pair(wg, tab);
    const float gg[2] = {widen_lo(g2), widen_hi(g2)};
    const float cp[2] = {c0.x, c0.y};
    float c1[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const float keep = fg[k] * cp[k], add = ig[k] * gg[k];
        c1[k] = keep + add;
    }
    const uint32_t tc2 = ktanh_pair(narrow_pair(c1[0], c1[1]), tab);
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
    return launch_grad<GRAD_TANH>(dy, y, dx, n, stream);
}

extern "C" ktanh_status_t ksigmoid_backward(const uint16_t *dy, const uint16_t *s, uint16_t *dx,
                                            size_t n, ktanh_stream_t stream)
{
    return launch_grad<GRAD_SIGMOID>(dy, s, dx, n, stream);
}

extern "C" ktanh_status_t kswish_backward(const uint16_t *dy, const uint16_t *x, uint16_t *dx,
                                          size_t n, const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    return launch_grad_from_input<GRAD_SWISH>(dy, x, dx, n, lut, stream);
}

extern "C" ktanh_status_t kgelu_backward(const uint16_t *dy, const uint16_t *x, uint16_t *dx,
                                         size_t n, const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    return launch_grad_from_input<GRAD_GELU>(dy, x, dx, n, lut, stream);
}

extern "C" ktanh_status_t ktanh_f32_backward(const float *dy, const float *y, float *dx, size_t n,
                                             ktanh_stream_t stream)
{
    return launch_grad_f32<GF_TANH>(dy, y, dx, n, nullptr, stream);
}

extern "C" ktanh_status_t ksigmoid_f32_backward(const float *dy, const float *s, float *dx, size_t n,
                                                ktanh_stream_t stream)
{
    return launch_grad_f32<GF_SIGMOID>(dy, s, dx, n, nullptr, stream);
}

extern "C" ktanh_status_t kswish_f32_backward(const float *dy, const float *x, float *dx, size_t n,
                                              const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    return launch_grad_f32<GF_SWISH>(dy, x, dx, n, lut, stream);
}

extern "C" ktanh_status_t kgelu_f32_backward(const float *dy, const float *x, float *dx, size_t n,
                                             const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    return launch_grad_f32<GF_GELU>(dy, x, dx, n, lut, stream);
}

extern "C" ktanh_status_t klstm_cell_backward(const uint16_t *gates, const float *c_prev,
                                              const uint16_t *dh, const float *dc_next,
                                              uint16_t *dgates, float *dc_prev, size_t B, size_t H,
                                              const ktanh_lut_t *lut, ktanh_stream_t stream)
{
    if (B == 0 || H == 0) return KT_OK;
    if (gates == nullptr || c_prev == nullptr || dh == nullptr || dc_next == nullptr ||
        dgates == nullptr || dc_prev == nullptr)
        return KT_ERR_NULL;
    if (H % 8 != 0) return KT_ERR_SHAPE;
    if (B > ((size_t)1 << 40) || H > ((size_t)1 << 40)) return KT_ERR_SHAPE;
    const uintptr_t mis = reinterpret_cast<uintptr_t>(gates) | reinterpret_cast<uintptr_t>(c_prev) |
                          reinterpret_cast<uintptr_t>(dh) | reinterpret_cast<uintptr_t>(dc_next) |
                          reinterpret_cast<uintptr_t>(dgates) | reinterpret_cast<uintptr_t>(dc_prev);
    if (mis & 15) return KT_ERR_ALIGN;
    KtLutPack pack;
    const ktanh_status_t st = kt_pack_lut_bf16(lut, &pack);
    if (st != KT_OK) return st;
    const unsigned long long n_pairs = (unsigned long long)B * (H / 2);
    if (n_pairs >= (1ull << 28)) return KT_ERR_SHAPE;  // word indices inside [B][4H] fit 32 bits
    const unsigned long long blocks = (n_pairs + kCellBlock - 1) / kCellBlock;
    return launch_checked(lstm_cell_backward_kernel, (unsigned)blocks, kCellBlock, stream,
                          reinterpret_cast<const uint32_t *>(gates),
                          reinterpret_cast<const float2 *>(c_prev),
                          reinterpret_cast<const uint32_t *>(dh),
                          reinterpret_cast<const float2 *>(dc_next),
                          reinterpret_cast<uint32_t *>(dgates), reinterpret_cast<float2 *>(dc_prev),
                          (unsigned)n_pairs, (unsigned)(H / 2), pack);
}
