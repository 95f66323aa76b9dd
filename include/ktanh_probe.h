/*
 * libktanh_probe -- measurement yardsticks for libktanh.  NOT operations of the paper and not part
 * of the product library: a separate shared object that a benchmark loads next to libktanh to see
 * what the memory system allows for the launch shape of the element-wise entry points (one
 * wavefront per block, one 128-bit vector per lane, the same load and store policies).
 *
 * Conventions as in ktanh.h: device pointers owned by the caller, `stream` a hipStream_t, calls only
 * enqueue, nothing is allocated or kept, errors are returned (ktanh_status_t) before any launch.
 */
#ifndef KTANH_PROBE_H
#define KTANH_PROBE_H

#include "ktanh.h"

#ifdef __cplusplus
extern "C" {
#endif

/* The launch of ktanh_bf16 with the arithmetic taken out: copies n 16-bit elements (same peeling of
 * unaligned heads and tails, same tiles).  in, out: device, n elements each, 2-byte aligned;
 * out == in allowed. */
ktanh_status_t ktanh_probe_copy(const uint16_t *in, uint16_t *out, size_t n, ktanh_stream_t stream);

/* The loads of that launch alone: reads n_bytes from `in` and writes nothing (a store guarded by a
 * test on the data, which keeps the loads in the code, would land inside `sink`).  in: device,
 * 1 KiB aligned, n_bytes a multiple of 16; sink: device, 1 KiB of scratch, 16-byte aligned. */
ktanh_status_t ktanh_probe_read(const void *in, void *sink, size_t n_bytes, ktanh_stream_t stream);

/* The stores of that launch alone: fills n_bytes at `out` with the BFloat16 pattern of 1.0.
 * out: device, 1 KiB aligned, n_bytes a multiple of 16. */
ktanh_status_t ktanh_probe_write(void *out, size_t n_bytes, ktanh_stream_t stream);

/* The same two with 512-thread blocks (eight wavefronts, one vector per lane): the launch shape of
 * the library asks the dispatcher for one block per KiB, which bounds a launch that only reads or
 * only writes; these show what the memory system itself gives to each direction.  Arguments as above. */
ktanh_status_t ktanh_probe_read_wide(const void *in, void *sink, size_t n_bytes, ktanh_stream_t stream);
ktanh_status_t ktanh_probe_write_wide(void *out, size_t n_bytes, ktanh_stream_t stream);

/* The launch of klstm_cell with the arithmetic taken out: the same loads (four gate words per lane
 * and step, prefetched the same number of steps ahead), stores, waits and loop.  Output word (t, b, j)
 * of h_out, taken as 32 bits over two neighbouring cells, is the XOR of the step's four gate words
 * and the bits of c_in[b][2j]; c_out = c_in.  Arguments, shapes, alignment and errors as klstm_cell. */
ktanh_status_t ktanh_probe_lstm(const uint16_t *gates, const float *c_in, float *c_out,
                                uint16_t *h_out, size_t T, size_t B, size_t H, ktanh_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* KTANH_PROBE_H */
