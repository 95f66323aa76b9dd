// libktanh: the entry points of the fused LSTM-cell element-wise kernel.
#include "ktanh_lstm_impl.h"

using namespace ktanh_device;

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
