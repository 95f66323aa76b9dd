/*
 * libktanh -- K-TanH (arXiv:1909.07729) and the activations derived from it, as HIP kernels for
 * AMD MI355X (gfx950) behind a plain C ABI.
 *
 * Conventions shared by every entry point
 *   - Tensor pointers (`in`, `out`, `gates`, `c_in`, `c_out`, `h_out`) are DEVICE pointers owned
 *     by the caller.  The library allocates nothing, frees nothing and keeps no pointer after the
 *     call returns.
 *   - `lut` is a HOST pointer to the 96-byte parameter table; it is read during the call and
 *     travels to the GPU inside the kernel arguments.  NULL selects the paper's Table 1.
 *   - `stream` is a hipStream_t passed as void*; NULL is the default stream.  Calls only enqueue
 *     work: they return without synchronising and may be issued from several host threads.  The
 *     library keeps nothing between calls except the fitted 64-interval table, computed once per
 *     process on first use.
 *   - BFloat16 tensors are arrays of uint16_t bit patterns (s:1, E:8, M:7); Float32 tensors of
 *     K-TanH are arrays of uint32_t bit patterns (s:1, E:8, M:23).  Tensors are dense and 1-D as
 *     far as the library is concerned (any contiguous shape works).
 *   - `out == in` (and `c_out == c_in`) is allowed; any other overlap is undefined.
 *   - Pointers must be aligned to their element size (else KT_ERR_ALIGN); nothing more is
 *     required.  The body always runs on 128-bit accesses: the elements before the output's first
 *     16-byte boundary and after its last are peeled, and an input that is not congruent to the
 *     output modulo 16 bytes is read with unaligned 128-bit loads (measured within a few per cent
 *     of the aligned case).  Results are identical.
 *   - n == 0 (or T, B or H == 0) returns KT_OK without launching anything.
 *   - Errors are returned, never thrown; nothing is launched when an argument is rejected.  A
 *     failed launch is reported as KT_ERR_HIP.
 */
#ifndef KTANH_H
#define KTANH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KTANH_INTERVALS 32

/* The three parameter tables T_E, T_r, T_b of Algorithm 1, 32 entries each (Table 1).
 * Entry t serves the interval whose index string is t = (2 LSBs of E_i) << 3 | (3 MSBs of M_i):
 * t = 8..15 covers [0.25, 0.5), 16..23 [0.5, 1), 24..31 [1, 2), 0..7 [2, 4). */
typedef struct ktanh_lut {
    uint8_t E[KTANH_INTERVALS]; /* biased output exponent E_t, 1..254                   */
    uint8_t r[KTANH_INTERVALS]; /* right shift r_t applied to the input mantissa, 0..7  */
    int8_t  b[KTANH_INTERVALS]; /* signed offset b_t added to the shifted mantissa      */
} ktanh_lut_t;

typedef void *ktanh_stream_t; /* a hipStream_t */

typedef enum ktanh_status {
    KT_OK = 0,
    KT_ERR_NULL = 1,  /* a required pointer is NULL                                       */
    KT_ERR_ALIGN = 2, /* a tensor pointer is not aligned to its element size              */
    KT_ERR_LUT = 3,   /* the table fails ktanh_lut_validate                               */
    KT_ERR_SHAPE = 4, /* klstm_cell: H not a multiple of 8; any entry point: tensor too large
                         (one call covers fewer than 2^26 wavefront tiles of 1 KiB of output,
                         i.e. just under 64 GiB; the LSTM cell fewer than 2^29 cells per step) */
    KT_ERR_HIP = 5    /* the HIP runtime refused the launch                               */
} ktanh_status_t;

/* Human-readable name of a status code; static storage. */
const char *ktanh_status_string(ktanh_status_t status);

/* Table 1 of the paper (optimised parameters for BFloat16 inputs).  Static storage: never free
 * it, never write through it. */
const ktanh_lut_t *ktanh_default_lut(void);

/* Checks that a table cannot overflow or underflow the 7-bit output mantissa, which is what the
 * bounds b_min and b_max of Section 2.4 (eq. (2)) guarantee for a fitted table: for every entry,
 * 1 <= E <= 254, 0 <= r <= 7, and 0 <= (M >> r) + b <= 127 for all 16 mantissas M of its interval.
 * Host-only; `lut` is a host pointer.  Returns KT_OK, KT_ERR_NULL or KT_ERR_LUT. */
ktanh_status_t ktanh_lut_validate(const ktanh_lut_t *lut);

/* K-TanH on BFloat16 (Algorithm 1; thresholds and index of Section 2.3):
 *   |x| <  0.25 (T1)                      -> x unchanged (zeros and subnormals included)
 *   |x| >= 4    (beyond T2 = 3.75 on the 8 exponent + 3 mantissa bits the test inspects;
 *                +-Inf included)          -> +-1
 *   otherwise                             -> (s_i, E_t, (M_i >> r_t) + b_t)
 *   NaN                                   -> the same NaN with its quiet bit set
 * in, out: device, n elements each. */
ktanh_status_t ktanh_bf16(const uint16_t *in, uint16_t *out, size_t n, const ktanh_lut_t *lut,
                          ktanh_stream_t stream);

/* K-TanH on Float32 (Algorithm 1; the paper states the method carries over to Float32 and gives
 * parameters for BFloat16 only): same thresholds and index on the leading bits, the 8-bit
 * parameters act on the 23-bit mantissa as M_o = (M_i >> r_t) + b_t * 2^16.  Truncating input and
 * output to their top 16 bits gives exactly ktanh_bf16.  in, out: device, n elements each. */
ktanh_status_t ktanh_f32(const uint32_t *in, uint32_t *out, size_t n, const ktanh_lut_t *lut,
                         ktanh_stream_t stream);

/* Activations derived from TanH (Section 1), BFloat16 in and out, n elements each, device.
 * K below is ktanh_bf16 applied to the BFloat16 rounding (nearest even) of its argument; all other
 * arithmetic is IEEE Float32, one rounding per operation, the result rounded to BFloat16 (nearest
 * even).  NaN in gives NaN out (which NaN is unspecified).
 *   ksigmoid(x) = 0.5 * K(0.5 x) + 0.5
 *   kswish(x)   = x * (0.5 * K(0.5 x) + 0.5)               (the Float32 Sigmoid, not re-rounded)
 *   kgelu(x)    = (0.5 x) * (1 + K(c * (x + a * ((x*x)*x)))),  a = 0.044715f, c = sqrt(2/pi) as float
 */
ktanh_status_t ksigmoid(const uint16_t *in, uint16_t *out, size_t n, const ktanh_lut_t *lut,
                        ktanh_stream_t stream);
ktanh_status_t kswish(const uint16_t *in, uint16_t *out, size_t n, const ktanh_lut_t *lut,
                      ktanh_stream_t stream);
ktanh_status_t kgelu(const uint16_t *in, uint16_t *out, size_t n, const ktanh_lut_t *lut,
                     ktanh_stream_t stream);

/* ---- 64-interval variant ------------------------------------------------------------------------
 * Section 2.4 (last paragraph): the parameters are 8-bit, so 64 intervals fit where AVX512 held 32
 * 16-bit values.  Index t = (2 LSBs of E_i) << 4 | (4 MSBs of M_i); t = 16..31 covers [0.25, 0.5),
 * 32..47 [0.5, 1), 48..63 [1, 2), 0..15 [2, 4).  Thresholds and everything else as in Algorithm 1. */
#define KTANH_INTERVALS64 64

typedef struct ktanh_lut64 {
    uint8_t E[KTANH_INTERVALS64];
    uint8_t r[KTANH_INTERVALS64];
    int8_t  b[KTANH_INTERVALS64];
} ktanh_lut64_t;

/* Offline parameter fit of Section 2.4 (Steps 1-3: common output exponent per interval, then the
 * (r, b) that minimise eq. (1) under the overflow bounds b_min, b_max of eq. (2)), for BFloat16
 * inputs.  Host-only, double precision, microseconds; `out` is a host pointer the caller owns.
 * ktanh_fit_lut reproduces Table 1; ktanh_fit_lut64 produces the 64-interval tables;
 * ktanh_fit_lut_bmin0 solves the same problem with b_min = 0, the deliberately sub-optimal
 * parameters of the ablation study in Section 3 (a valid table: pass it as `lut` to see its effect).
 * Returns KT_OK or KT_ERR_NULL. */
ktanh_status_t ktanh_fit_lut(ktanh_lut_t *out);
ktanh_status_t ktanh_fit_lut64(ktanh_lut64_t *out);
ktanh_status_t ktanh_fit_lut_bmin0(ktanh_lut_t *out);

/* Same check as ktanh_lut_validate for a 64-interval table (8 mantissas per interval). */
ktanh_status_t ktanh_lut64_validate(const ktanh_lut64_t *lut);

/* K-TanH with a 64-interval table on BFloat16 / Float32: same contract as ktanh_bf16 / ktanh_f32.
 * `lut` == NULL selects the table ktanh_fit_lut64 produces (fitted once per process, on first use). */
ktanh_status_t ktanh64_bf16(const uint16_t *in, uint16_t *out, size_t n, const ktanh_lut64_t *lut,
                            ktanh_stream_t stream);
ktanh_status_t ktanh64_f32(const uint32_t *in, uint32_t *out, size_t n, const ktanh_lut64_t *lut,
                           ktanh_stream_t stream);

/* ksigmoid, kswish, kgelu and klstm_cell (declared below and above) with a 64-interval table: same
 * contracts, same operation sequences, K = ktanh64_bf16. */
ktanh_status_t ksigmoid64(const uint16_t *in, uint16_t *out, size_t n, const ktanh_lut64_t *lut,
                          ktanh_stream_t stream);
ktanh_status_t kswish64(const uint16_t *in, uint16_t *out, size_t n, const ktanh_lut64_t *lut,
                        ktanh_stream_t stream);
ktanh_status_t kgelu64(const uint16_t *in, uint16_t *out, size_t n, const ktanh_lut64_t *lut,
                       ktanh_stream_t stream);
ktanh_status_t klstm_cell64(const uint16_t *gates, const float *c_in, float *c_out, uint16_t *h_out,
                            size_t T, size_t B, size_t H, const ktanh_lut64_t *lut,
                            ktanh_stream_t stream);

/* ---- Float32 tensors -----------------------------------------------------------------------------
 * The Section 1 identities on Float32 data with the Float32 form of Algorithm 1 (ktanh_f32) inside;
 * nothing is rounded to BFloat16.  IEEE Float32, one rounding per operation, in this order:
 *   ksigmoid_f32(x) = 0.5 * Kf(0.5 x) + 0.5
 *   kswish_f32(x)   = x * (0.5 * Kf(0.5 x) + 0.5)
 *   kgelu_f32(x)    = (0.5 x) * (1 + Kf(c * (x + a * ((x*x)*x))))
 * in, out: device, n elements each, 4-byte aligned.
 * NaN in gives NaN out. */
ktanh_status_t ksigmoid_f32(const float *in, float *out, size_t n, const ktanh_lut_t *lut,
                            ktanh_stream_t stream);
ktanh_status_t kswish_f32(const float *in, float *out, size_t n, const ktanh_lut_t *lut,
                          ktanh_stream_t stream);
ktanh_status_t kgelu_f32(const float *in, float *out, size_t n, const ktanh_lut_t *lut,
                         ktanh_stream_t stream);
/* The same three with a 64-interval table (ktanh64_f32 inside); `lut` == NULL selects the fitted one. */
ktanh_status_t ksigmoid64_f32(const float *in, float *out, size_t n, const ktanh_lut64_t *lut,
                              ktanh_stream_t stream);
ktanh_status_t kswish64_f32(const float *in, float *out, size_t n, const ktanh_lut64_t *lut,
                            ktanh_stream_t stream);
ktanh_status_t kgelu64_f32(const float *in, float *out, size_t n, const ktanh_lut64_t *lut,
                           ktanh_stream_t stream);

/* K-TanH on BFloat16 inputs that arrive as Float32: each value is rounded to BFloat16 (nearest even)
 * and goes through ktanh_bf16 -- the conversion Section 2.5 leaves out of the paper's cycle count,
 * fused into the load (6 bytes of traffic per element instead of 4 + 4 + 4).
 * in: device, n Float32, 4-byte aligned; out: device, n BFloat16, 2-byte aligned (any such pair:
 * the body reads 128 bits and writes 64 bits per lane from wherever `out` reaches an 8-byte boundary).
 * NaN in gives NaN out (which NaN is unspecified). */
ktanh_status_t ktanh_f32_to_bf16(const float *in, uint16_t *out, size_t n, const ktanh_lut_t *lut,
                                 ktanh_stream_t stream);

/* Element-wise part of an LSTM cell with K-TanH non-linearities (the recurrent GNMT workload of
 * Section 3 is what it serves; Sigmoid as in Section 1), over T consecutive time steps whose gate
 * pre-activations are all given:
 *   gates [T][B][4H] BFloat16, device: each row holds the blocks i | f | g | o, H values each
 *   c_in  [B][H]     Float32,  device: cell state before the first step
 *   c_out [B][H]     Float32,  device: cell state after the last step (may be c_in)
 *   h_out [T][B][H]  BFloat16, device: hidden output of every step
 * Per cell and step, in Float32:  i, f, o = 0.5*K(0.5 g_.)+0.5;  g = K(g_g);
 *   c' = (f*c) + (i*g);  h' = bf16(o * K(bf16(c'))).   The state is carried in registers between
 * the T steps.  T == 1 is the ordinary per-step call of a recurrent network.
 * H must be a multiple of 8 (KT_ERR_SHAPE).  The kernel moves BFloat16 pairs and Float32 pairs:
 * gates and h_out must be 4-byte aligned, c_in and c_out 8-byte aligned (KT_ERR_ALIGN). */
ktanh_status_t klstm_cell(const uint16_t *gates, const float *c_in, float *c_out, uint16_t *h_out,
                          size_t T, size_t B, size_t H, const ktanh_lut_t *lut,
                          ktanh_stream_t stream);

/* ---- Gradients ------------------------------------------------------------------------------------
 * Section 3 trains GNMT through K-TanH; the paper does not say how the gradient is formed.  These
 * entry points use the derivative identities of TanH and Sigmoid on the forward outputs:
 *   ktanh_bf16_backward:  dx = bf16( dy * (1 - y*y) ),      y = forward K-TanH output
 *   ksigmoid_backward:    dx = bf16( dy * (s * (1 - s)) ),  s = forward Sigmoid output
 * BFloat16 tensors of n elements, device; Float32 arithmetic, one rounding per operation, result
 * rounded to nearest even.  dx may alias dy or the forward output.  No table is involved. */
ktanh_status_t ktanh_bf16_backward(const uint16_t *dy, const uint16_t *y, uint16_t *dx, size_t n,
                                   ktanh_stream_t stream);
ktanh_status_t ksigmoid_backward(const uint16_t *dy, const uint16_t *s, uint16_t *dx, size_t n,
                                 ktanh_stream_t stream);

/* Gradients of the Swish and GELU identities of Section 1 with the K-TanH value in place of TanH,
 * from the forward INPUT x (the value is rebuilt exactly as kswish / kgelu form it):
 *   kswish_backward:  dx = bf16( dy * (s + x*(s*(1 - s))) ),                      s = Sigmoid(x)
 *   kgelu_backward:   dx = bf16( dy * (0.5*(1 + t) + (0.5*x)*((1 - t*t)*(c*(1 + a3*(x*x))))) ),
 *                     t = K(bf16(c*(x + a*x^3))), a = 0.044715, a3 = 0.134145 (= 3a), c = sqrt(2/pi)
 * BFloat16 tensors of n elements, device; `lut` as for the forward calls (host pointer, NULL =
 * Table 1).  Float32 arithmetic, one rounding per operation in the order written, result rounded
 * to nearest even.  Non-finite intermediates behave as the operations give (x*x overflows beyond
 * |x| = 1.8e19 and the GELU slope is then NaN).  dx may alias dy or x. */
ktanh_status_t kswish_backward(const uint16_t *dy, const uint16_t *x, uint16_t *dx, size_t n,
                               const ktanh_lut_t *lut, ktanh_stream_t stream);
ktanh_status_t kgelu_backward(const uint16_t *dy, const uint16_t *x, uint16_t *dx, size_t n,
                              const ktanh_lut_t *lut, ktanh_stream_t stream);

/* The same four gradients on Float32 tensors (n elements each, device, 4-byte aligned): the
 * formulas above with nothing rounded to BFloat16 and, inside Swish and GELU, the Float32 K-TanH of ksigmoid_f32 / kgelu_f32.
 * y, s: forward outputs of ktanh_f32 / ksigmoid_f32 as Float32 values; x: forward input.
 * dx may alias dy or the other input. */
ktanh_status_t ktanh_f32_backward(const float *dy, const float *y, float *dx, size_t n,
                                  ktanh_stream_t stream);
ktanh_status_t ksigmoid_f32_backward(const float *dy, const float *s, float *dx, size_t n,
                                     ktanh_stream_t stream);
ktanh_status_t kswish_f32_backward(const float *dy, const float *x, float *dx, size_t n,
                                   const ktanh_lut_t *lut, ktanh_stream_t stream);
ktanh_status_t kgelu_f32_backward(const float *dy, const float *x, float *dx, size_t n,
                                  const ktanh_lut_t *lut, ktanh_stream_t stream);

/* One klstm_cell step backwards.  The forward activations are recomputed from the gate
 * pre-activations with K-TanH exactly as klstm_cell forms them (i, f, o, g, c' = f*c + i*g,
 * tc = K(bf16(c'))); then, in Float32, one rounding per operation:
 *   do = dh*tc;   dc = dc_next + (dh*o)*(1 - tc*tc);
 *   di = dc*g;  df = dc*c_prev;  dg = dc*i;  dc_prev = dc*f;
 *   dgates = bf16( di*(i*(1-i)) | df*(f*(1-f)) | dg*(1 - g*g) | do*(o*(1-o)) )
 *   gates   [B][4H] BFloat16 (i|f|g|o), device     c_prev  [B][H] Float32, device
 *   dh      [B][H]  BFloat16, device               dc_next [B][H] Float32, device
 *   dgates  [B][4H] BFloat16, device, out          dc_prev [B][H] Float32, device, out (may be dc_next)
 * H must be a multiple of 8 (KT_ERR_SHAPE); gates, dh and dgates 4-byte aligned, c_prev, dc_next and
 * dc_prev 8-byte aligned (KT_ERR_ALIGN). */
ktanh_status_t klstm_cell_backward(const uint16_t *gates, const float *c_prev, const uint16_t *dh,
                                   const float *dc_next, uint16_t *dgates, float *dc_prev, size_t B,
                                   size_t H, const ktanh_lut_t *lut, ktanh_stream_t stream);


/* ---- Comparison approximants ---------------------------------------------------------------------
 * The rational Pade approximants of Section 2 ("Pade rational Polynomial"), which Table 2 sets
 * against K-TanH: the quotient of two polynomials whose value and first p+q derivatives at zero are
 * TanH's, scaled to integer coefficients:
 *   kpade32_bf16:  x (15 + x^2) / (15 + 6 x^2)                      evaluated on min(|x|, 4), capped at 1
 *   kpade78_bf16:  x (2027025 + 270270 x^2 + 6930 x^4 + 36 x^6)
 *                  / (2027025 + 945945 x^2 + 51975 x^4 + 630 x^6 + x^8)   evaluated on min(|x|, 5.5)
 * (the first grows without bound, the second peaks at |x| = 5.70 and decays: hence the cut-offs, which
 * the paper does not give).  BFloat16 in and out, n elements each, device; Float32 arithmetic, one
 * rounding per operation, Horner's scheme in x^2 on |x|, correctly rounded division, the sign put
 * back, the result rounded to nearest even; a NaN is returned quieted.  No table is involved.
 * Same conventions (alignment, aliasing, sizes, errors) as ktanh_bf16. */
ktanh_status_t kpade32_bf16(const uint16_t *in, uint16_t *out, size_t n, ktanh_stream_t stream);
ktanh_status_t kpade78_bf16(const uint16_t *in, uint16_t *out, size_t n, ktanh_stream_t stream);

/* Table 2's rows "Taylor approx degree 2" and "degree 3".  The paper names the method (Section 1) and
 * prints two error figures per row, but neither partition nor expansion point.  Built here on
 * K-TanH's own terms: the regions of Algorithm 1 (|x| below T1 = 0.25 is returned as it is, |x| from
 * 4.0 on gives +-1) and, in between, the 32 intervals that Table 1's index t names (2 low exponent
 * bits, 3 high mantissa bits); on each the Taylor polynomial of TanH of that degree about the
 * interval's midpoint a_t, sum_k TanH^(k)(a_t)/k! (|x| - a_t)^k.  A table entry is thus 3 or 4 Float32
 * coefficients (formed in double precision, then rounded) in place of K-TanH's three small integers.
 * BFloat16 in and out, n elements each, device; Float32 arithmetic, Horner's scheme, one rounding per
 * operation, the sign put back, the result rounded to nearest even; a NaN is returned quieted.  The
 * table is fixed: there is no table argument.  This reading is far more accurate than the figures
 * Table 2 prints for these rows (its error is that of the BFloat16 result, half a step).
 * Same conventions (alignment, aliasing, sizes, errors) as ktanh_bf16. */
ktanh_status_t ktaylor2_bf16(const uint16_t *in, uint16_t *out, size_t n, ktanh_stream_t stream);
ktanh_status_t ktaylor3_bf16(const uint16_t *in, uint16_t *out, size_t n, ktanh_stream_t stream);

/* The gradients that read a table, with a 64-interval table (Section 2.4, last paragraph) inside:
 * the same formulas and operation order with K = ktanh64_bf16 (ktanh64_f32 on Float32 tensors).
 * `lut` == NULL selects the fitted 64-interval table.  (ktanh_bf16_backward, ksigmoid_backward and
 * their Float32 forms take the forward output and read no table: they serve both table sizes.) */
ktanh_status_t kswish64_backward(const uint16_t *dy, const uint16_t *x, uint16_t *dx, size_t n,
                                 const ktanh_lut64_t *lut, ktanh_stream_t stream);
ktanh_status_t kgelu64_backward(const uint16_t *dy, const uint16_t *x, uint16_t *dx, size_t n,
                                const ktanh_lut64_t *lut, ktanh_stream_t stream);
ktanh_status_t kswish64_f32_backward(const float *dy, const float *x, float *dx, size_t n,
                                     const ktanh_lut64_t *lut, ktanh_stream_t stream);
ktanh_status_t kgelu64_f32_backward(const float *dy, const float *x, float *dx, size_t n,
                                    const ktanh_lut64_t *lut, ktanh_stream_t stream);
ktanh_status_t klstm_cell64_backward(const uint16_t *gates, const float *c_prev, const uint16_t *dh,
                                     const float *dc_next, uint16_t *dgates, float *dc_prev, size_t B,
                                     size_t H, const ktanh_lut64_t *lut, ktanh_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* KTANH_H */
