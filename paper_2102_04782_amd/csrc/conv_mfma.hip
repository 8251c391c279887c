// int8 MFMA convolution kernels (placeholder: nothing supported yet, direct kernels are used).
#include "daq_internal.h"

namespace daq {
bool bwd_filter_mfma_supported(const daq_conv_desc&) { return false; }
size_t bwd_filter_mfma_ws_bytes(const daq_conv_desc&) { return 0; }
daq_status conv_bwd_filter_mfma(const daq_conv_desc&, const int8_t*, const float*, const int8_t*, const float*, float*,
                                int32_t*, void*, hipStream_t) { return DAQ_ERR_UNSUPPORTED; }
bool bwd_data_mfma_supported(const daq_conv_desc&) { return false; }
daq_status conv_bwd_data_mfma(const daq_conv_desc&, const int8_t*, const float*, const int8_t*, const float*, float*,
                              int32_t*, hipStream_t) { return DAQ_ERR_UNSUPPORTED; }
bool fwd_mfma_supported(const daq_conv_desc&) { return false; }
daq_status conv_fwd_mfma(const daq_conv_desc&, const int8_t*, const int8_t*, const float*, const float*, float*,
                         int32_t*, hipStream_t) { return DAQ_ERR_UNSUPPORTED; }
}  // namespace daq
