// A consumer of the C ABI with no Python and no torch in the loop: device memory from the HIP
// runtime, the library's entry points on a stream of its own, results compared on the host with
// the CPU checker under oracle/ (linked as a shared library; test infrastructure).
// Built by __graft_entry__.build(), run by tests/test_gpu_parity.py.  Exit status 0 = all match.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "ktanh.h"

extern "C" {
typedef struct {
    uint8_t E[32];
    uint8_t r[32];
    int8_t b[32];
} oracle_lut;
void oracle_table1(oracle_lut *lut);
void oracle_ktanh_bf16(const uint16_t *in, uint16_t *out, size_t n, const oracle_lut *lut);
void oracle_ksigmoid(const uint16_t *in, uint16_t *out, size_t n, const oracle_lut *lut);
void oracle_kswish(const uint16_t *in, uint16_t *out, size_t n, const oracle_lut *lut);
void oracle_kgelu(const uint16_t *in, uint16_t *out, size_t n, const oracle_lut *lut);
void oracle_ktanh_f32(const uint32_t *in, uint32_t *out, size_t n, const oracle_lut *lut);
void oracle_klstm_cell(const uint16_t *gates, const float *c_in, float *c_out, uint16_t *h_out,
                       size_t T, size_t B, size_t H, const oracle_lut *lut);
}

namespace {

#define HIP_OK(call)                                                                     \
    do {                                                                                 \
        hipError_t e_ = (call);                                                          \
        if (e_ != hipSuccess) {                                                          \
            std::fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));              \
            std::exit(2);                                                                \
        }                                                                                \
    } while (0)

#define KT_OK_OR_DIE(call)                                                               \
    do {                                                                                 \
        ktanh_status_t s_ = (call);                                                      \
        if (s_ != KT_OK) {                                                               \
            std::fprintf(stderr, "%s: %s\n", #call, ktanh_status_string(s_));            \
            std::exit(3);                                                                \
        }                                                                                \
    } while (0)

uint32_t next_random(uint32_t &state)  // xorshift32: any seeded stream of bits will do here
{
    state ^= state << 13;
    state ^= state >> 17;
    state ^= state << 5;
    return state;
}

bool is_nan_bf16(uint16_t v) { return (v & 0x7FFF) > 0x7F80; }

// Bit-exact, except that a NaN only has to be a NaN (the derived activations do not fix which).
size_t mismatches_bf16(const std::vector<uint16_t> &got, const std::vector<uint16_t> &want, bool exact_nan)
{
    size_t bad = 0;
    for (size_t i = 0; i < got.size(); ++i) {
        if (!exact_nan && is_nan_bf16(want[i])) {
            bad += !is_nan_bf16(got[i]);
        } else {
            bad += got[i] != want[i];
        }
    }
    return bad;
}

template <class T>
struct DeviceBuffer {
    T *ptr = nullptr;
    explicit DeviceBuffer(size_t n) { HIP_OK(hipMalloc(reinterpret_cast<void **>(&ptr), n * sizeof(T) + 16)); }
    ~DeviceBuffer() { (void)hipFree(ptr); }
};

}  // namespace

int main()
{
    oracle_lut table;
    oracle_table1(&table);
    if (std::memcmp(&table, ktanh_default_lut(), sizeof table) != 0) {
        std::fprintf(stderr, "the library's Table 1 differs from the checker's\n");
        return 1;
    }
    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));
    size_t failures = 0;

    // every BFloat16 pattern, then 100,003 more drawn around the activation range
    uint32_t seed = 190907u;
    std::vector<uint16_t> x(65536 + 100003);
    for (size_t i = 0; i < 65536; ++i) x[i] = (uint16_t)i;
    for (size_t i = 65536; i < x.size(); ++i) {
        const uint32_t r = next_random(seed);
        x[i] = (uint16_t)(((r & 1u) << 15) | (0x3C00u + (r >> 8) % 0x0600u));  // |x| in [2^-7, 16)
    }
    const size_t n = x.size();
    DeviceBuffer<uint16_t> dx(n), dy(n);
    HIP_OK(hipMemcpyAsync(dx.ptr, x.data(), n * 2, hipMemcpyHostToDevice, stream));
    struct Op {
        const char *name;
        ktanh_status_t (*gpu)(const uint16_t *, uint16_t *, size_t, const ktanh_lut_t *, ktanh_stream_t);
        void (*cpu)(const uint16_t *, uint16_t *, size_t, const oracle_lut *);
        bool exact_nan;
    };
    const Op ops[] = {{"ktanh_bf16", ktanh_bf16, oracle_ktanh_bf16, true},
                      {"ksigmoid", ksigmoid, oracle_ksigmoid, false},
                      {"kswish", kswish, oracle_kswish, false},
                      {"kgelu", kgelu, oracle_kgelu, false}};
    std::vector<uint16_t> got(n), want(n);
    for (const Op &op : ops) {
        // aligned, then shifted by one element on both sides (ragged head and tail)
        for (size_t shift = 0; shift < 2; ++shift) {
            const size_t m = n - 2 * shift;
            KT_OK_OR_DIE(op.gpu(dx.ptr + shift, dy.ptr + shift, m, nullptr, stream));
            got.assign(m, 0);
            want.assign(m, 0);
            HIP_OK(hipMemcpyAsync(got.data(), dy.ptr + shift, m * 2, hipMemcpyDeviceToHost, stream));
            HIP_OK(hipStreamSynchronize(stream));
            op.cpu(x.data() + shift, want.data(), m, &table);
            const size_t bad = mismatches_bf16(got, want, op.exact_nan);
            std::printf("%-10s shift %zu: %zu mismatches of %zu\n", op.name, shift, bad, m);
            failures += bad;
        }
    }

    // Float32: random bit patterns
    {
        const size_t nf = (1u << 20) + 3;
        std::vector<uint32_t> u(nf), gotf(nf), wantf(nf);
        for (uint32_t &v : u) v = next_random(seed);
        DeviceBuffer<uint32_t> du(nf), dv(nf);
        HIP_OK(hipMemcpyAsync(du.ptr, u.data(), nf * 4, hipMemcpyHostToDevice, stream));
        KT_OK_OR_DIE(ktanh_f32(du.ptr, dv.ptr, nf, nullptr, stream));
        HIP_OK(hipMemcpyAsync(gotf.data(), dv.ptr, nf * 4, hipMemcpyDeviceToHost, stream));
        HIP_OK(hipStreamSynchronize(stream));
        oracle_ktanh_f32(u.data(), wantf.data(), nf, &table);
        size_t bad = 0;
        for (size_t i = 0; i < nf; ++i) bad += gotf[i] != wantf[i];
        std::printf("%-10s          %zu mismatches of %zu\n", "ktanh_f32", bad, nf);
        failures += bad;
    }

    // LSTM cell: 11 steps in one call, state in place
    {
        const size_t T = 11, B = 3, H = 72;
        std::vector<uint16_t> gates(T * B * 4 * H), h_got(T * B * H), h_want(T * B * H);
        std::vector<float> c0(B * H), c_got(B * H), c_want(B * H);
        for (uint16_t &g : gates) {
            const uint32_t r = next_random(seed);
            g = (uint16_t)(((r & 1u) << 15) | (0x3D00u + (r >> 8) % 0x0400u));
        }
        for (float &c : c0) c = (float)((int)(next_random(seed) % 4001u) - 2000) / 1000.0f;
        DeviceBuffer<uint16_t> dg(gates.size()), dh(h_got.size());
        DeviceBuffer<float> dc(c0.size());
        HIP_OK(hipMemcpyAsync(dg.ptr, gates.data(), gates.size() * 2, hipMemcpyHostToDevice, stream));
        HIP_OK(hipMemcpyAsync(dc.ptr, c0.data(), c0.size() * 4, hipMemcpyHostToDevice, stream));
        KT_OK_OR_DIE(klstm_cell(dg.ptr, dc.ptr, dc.ptr, dh.ptr, T, B, H, nullptr, stream));
        HIP_OK(hipMemcpyAsync(h_got.data(), dh.ptr, h_got.size() * 2, hipMemcpyDeviceToHost, stream));
        HIP_OK(hipMemcpyAsync(c_got.data(), dc.ptr, c_got.size() * 4, hipMemcpyDeviceToHost, stream));
        HIP_OK(hipStreamSynchronize(stream));
        oracle_klstm_cell(gates.data(), c0.data(), c_want.data(), h_want.data(), T, B, H, &table);
        size_t bad = mismatches_bf16(h_got, h_want, false);
        bad += std::memcmp(c_got.data(), c_want.data(), c_got.size() * 4) != 0;
        std::printf("%-10s          %zu mismatches\n", "klstm_cell", bad);
        failures += bad;
    }

    HIP_OK(hipStreamDestroy(stream));
    if (failures != 0) {
        std::printf("FAILED: %zu mismatches\n", failures);
        return 1;
    }
    std::printf("all match\n");
    return 0;
}
