// Entry points of the three convolutions: argument validation and kernel selection.
#include "daq_internal.h"
#include "dw_tail.h"

using namespace daq;

namespace {
bool ws_ok(const void* ws, size_t have, size_t need) { return ws && have >= need && ((uintptr_t)ws & 255u) == 0; }
// int8 buffers are read and written as 16-byte vectors, fp32 tensors at least as dwords
bool a16(const void* p) { return ((uintptr_t)p & 15u) == 0; }
bool a4(const void* p) { return ((uintptr_t)p & 3u) == 0; }
}  // namespace

extern "C" daq_status daq_conv_fwd_int8_ex(const daq_conv_desc* desc, const float* X, const float* W, int8_t* qx_nhwc,
                                           int8_t* qx_cnhw, int8_t* qw_packed, float* s_x, float* s_w, float* Y,
                                           int32_t* acc_out, daq_schedule schedule, void* workspace,
                                           size_t workspace_bytes, void* stream) {
    if (!desc_valid(desc) || !X || !W || !qx_nhwc || !qx_cnhw || !qw_packed || !s_x || !s_w || !Y)
        return DAQ_ERR_INVALID_ARG;
    if (!a4(X) || !a4(W) || !a16(qx_nhwc) || !a16(qx_cnhw) || !a16(qw_packed) || !a16(Y) || !a16(acc_out))
        return DAQ_ERR_INVALID_ARG;
    if (schedule != DAQ_SCHEDULE_AUTO && schedule != DAQ_SCHEDULE_THREE_SWEEPS && schedule != DAQ_SCHEDULE_EARLY_COPY &&
        schedule != DAQ_SCHEDULE_CHANNEL_RESIDENT)   // the last has no forward form: one sweep per layout
        return DAQ_ERR_INVALID_ARG;
    const size_t need = daq_workspace_bytes(DAQ_OP_CONV_FWD, desc);
    if (need == 0) return DAQ_ERR_UNSUPPORTED;
    if (!ws_ok(workspace, workspace_bytes, need)) return DAQ_ERR_WORKSPACE;
    daq_status rc = quantize_activation_check(*desc, X);   // nothing is launched for a tensor the quantizers cannot take
    if (rc != DAQ_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    rc = quantize_activation(*desc, X, qx_nhwc, qx_cnhw, s_x, workspace, st, schedule);
    if (rc != DAQ_OK) return rc;
    rc = quantize_filter(*desc, W, qw_packed, s_w, workspace, st);
    if (rc != DAQ_OK) return rc;
    if (fwd_halo_supported(*desc)) return conv_fwd_halo(*desc, qx_nhwc, qw_packed, s_x, s_w, Y, acc_out, st);
    if (depthwise_fwd_supported(*desc)) return conv_fwd_depthwise(*desc, qx_cnhw, qw_packed, s_x, s_w, Y, acc_out, st);
    if (fwd_mfma_supported(*desc)) return conv_fwd_mfma(*desc, qx_nhwc, qw_packed, s_x, s_w, Y, acc_out, st);
    return conv_fwd_generic(*desc, qx_nhwc, qw_packed, s_x, s_w, Y, acc_out, st);
}

extern "C" daq_status daq_conv_fwd_int8(const daq_conv_desc* desc, const float* X, const float* W, int8_t* qx_nhwc,
                                        int8_t* qx_cnhw, int8_t* qw_packed, float* s_x, float* s_w, float* Y,
                                        int32_t* acc_out, void* workspace, size_t workspace_bytes, void* stream) {
    return daq_conv_fwd_int8_ex(desc, X, W, qx_nhwc, qx_cnhw, qw_packed, s_x, s_w, Y, acc_out, DAQ_SCHEDULE_AUTO, workspace,
                                workspace_bytes, stream);
}

extern "C" daq_status daq_conv_bwd_data_int8(const daq_conv_desc* desc, const int8_t* qg, const float* s_global,
                                             const int8_t* qw_packed, const float* s_w, float* dX, int32_t* acc_out,
                                             void* workspace, size_t workspace_bytes, void* stream) {
    if (!desc_valid(desc) || !qg || !s_global || !qw_packed || !s_w || !dX) return DAQ_ERR_INVALID_ARG;
    if (!a16(qg) || !a16(qw_packed) || !a16(dX) || !a16(acc_out)) return DAQ_ERR_INVALID_ARG;
    const size_t need = daq_workspace_bytes(DAQ_OP_CONV_BWD_DATA, desc);
    if (need == 0) return DAQ_ERR_UNSUPPORTED;
    if (!ws_ok(workspace, workspace_bytes, need)) return DAQ_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    if (bwd_data_halo_supported(*desc)) return conv_bwd_data_halo(*desc, qg, s_global, qw_packed, s_w, dX, acc_out, st);
    if (bwd_data_mfma_supported(*desc)) return conv_bwd_data_mfma(*desc, qg, s_global, qw_packed, s_w, dX, acc_out, st);
    if (depthwise_dx_supported(*desc)) return conv_bwd_data_depthwise(*desc, qg, s_global, qw_packed, s_w, dX, acc_out, st);
    return conv_bwd_data_generic(*desc, qg, s_global, qw_packed, s_w, dX, acc_out, st);
}

extern "C" daq_status daq_conv_bwd_filter_int8(const daq_conv_desc* desc, const int8_t* qx_cnhw, const float* s_x,
                                               const int8_t* vq, const float* s_chan, float* dW, int32_t* acc_out,
                                               void* workspace, size_t workspace_bytes, void* stream) {
    if (!desc_valid(desc) || !qx_cnhw || !s_x || !vq || !s_chan || !dW) return DAQ_ERR_INVALID_ARG;
    if (!a16(qx_cnhw) || !a16(vq) || !a4(dW) || !a4(acc_out)) return DAQ_ERR_INVALID_ARG;
    const size_t need = daq_workspace_bytes(DAQ_OP_CONV_BWD_FILTER, desc);
    if (need == 0) return DAQ_ERR_UNSUPPORTED;
    if (!ws_ok(workspace, workspace_bytes, need)) return DAQ_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    if (bwd_filter_lds_supported(*desc))
        return conv_bwd_filter_lds(*desc, qx_cnhw, s_x, vq, s_chan, dW, acc_out, workspace, st);
    if (bwd_filter_mfma_supported(*desc))
        return conv_bwd_filter_mfma(*desc, qx_cnhw, s_x, vq, s_chan, dW, acc_out, workspace, st);
    if (depthwise_dw_supported(*desc))
        return conv_bwd_filter_depthwise(*desc, qx_cnhw, s_x, vq, s_chan, dW, acc_out, workspace, st);
    return conv_bwd_filter_generic(*desc, qx_cnhw, s_x, vq, s_chan, dW, acc_out, st);
}

extern "C" daq_status daq_conv_bwd_int8(const daq_conv_desc* desc, const int8_t* qx_cnhw, const float* s_x,
                                        const int8_t* vq, const float* s_chan, float* dW, int32_t* dW_acc,
                                        const int8_t* qg, const float* s_global, const int8_t* qw_packed,
                                        const float* s_w, float* dX, int32_t* dX_acc, void* workspace,
                                        size_t workspace_bytes, void* stream) {
    if (!desc_valid(desc) || !qx_cnhw || !s_x || !vq || !s_chan || !dW || !qg || !s_global || !qw_packed || !s_w || !dX)
        return DAQ_ERR_INVALID_ARG;
    if (!a16(qx_cnhw) || !a16(vq) || !a4(dW) || !a4(dW_acc) || !a16(qg) || !a16(qw_packed) || !a16(dX) || !a16(dX_acc))
        return DAQ_ERR_INVALID_ARG;
    const size_t need_f = daq_workspace_bytes(DAQ_OP_CONV_BWD_FILTER, desc);
    const size_t need_d = daq_workspace_bytes(DAQ_OP_CONV_BWD_DATA, desc);
    if (need_f == 0 || need_d == 0) return DAQ_ERR_UNSUPPORTED;
    if (!ws_ok(workspace, workspace_bytes, need_f + need_d)) return DAQ_ERR_WORKSPACE;
    void* ws_d = static_cast<char*>(workspace) + need_f;   // need_f is a multiple of 256
    if (bwd_filter_lds_supported(*desc) && bwd_data_halo_supported(*desc)) {
        hipStream_t st = (hipStream_t)stream;
        DwTail tail{};
        const daq_status rc = conv_bwd_filter_lds(*desc, qx_cnhw, s_x, vq, s_chan, dW, dW_acc, workspace, st, &tail);
        if (rc != DAQ_OK) return rc;
        return conv_bwd_data_halo(*desc, qg, s_global, qw_packed, s_w, dX, dX_acc, st, tail.blocks > 0 ? &tail : nullptr);
    }
    const daq_status rc = daq_conv_bwd_filter_int8(desc, qx_cnhw, s_x, vq, s_chan, dW, dW_acc, workspace, need_f, stream);
    if (rc != DAQ_OK) return rc;
    return daq_conv_bwd_data_int8(desc, qg, s_global, qw_packed, s_w, dX, dX_acc, ws_d, need_d, stream);
}

extern "C" daq_status daq_conv_bwd_data_int8_bf16(const daq_conv_desc* desc, const int8_t* qg, const float* s_global,
                                                  const int8_t* qw_packed, const float* s_w, uint16_t* dX_bf16,
                                                  void* workspace, size_t workspace_bytes, void* stream) {
    if (!desc_valid(desc) || !qg || !s_global || !qw_packed || !s_w || !dX_bf16) return DAQ_ERR_INVALID_ARG;
    if (!a16(qg) || !a16(qw_packed) || !a16(dX_bf16)) return DAQ_ERR_INVALID_ARG;
    const size_t need = daq_workspace_bytes(DAQ_OP_CONV_BWD_DATA, desc);
    if (need == 0) return DAQ_ERR_UNSUPPORTED;
    if (!ws_ok(workspace, workspace_bytes, need)) return DAQ_ERR_WORKSPACE;
    // the kernels of daq_conv_bwd_data_int8, each with its narrow epilogue
    hipStream_t st = (hipStream_t)stream;
    float* out = reinterpret_cast<float*>(dX_bf16);
    if (bwd_data_halo_supported(*desc))
        return conv_bwd_data_halo(*desc, qg, s_global, qw_packed, s_w, out, nullptr, st, nullptr, true);
    if (bwd_data_mfma_supported(*desc)) return conv_bwd_data_mfma(*desc, qg, s_global, qw_packed, s_w, out, nullptr, st, true);
    if (depthwise_dx_supported(*desc))
        return conv_bwd_data_depthwise(*desc, qg, s_global, qw_packed, s_w, out, nullptr, st, false, true);
    return conv_bwd_data_generic(*desc, qg, s_global, qw_packed, s_w, out, nullptr, st, true);
}

extern "C" daq_status daq_conv_bwd_filter_int8_bf16(const daq_conv_desc* desc, const int8_t* qx_cnhw, const float* s_x,
                                                    const int8_t* vq, const float* s_chan, uint16_t* dW_bf16,
                                                    void* workspace, size_t workspace_bytes, void* stream) {
    if (!desc_valid(desc) || !qx_cnhw || !s_x || !vq || !s_chan || !dW_bf16) return DAQ_ERR_INVALID_ARG;
    if (!a16(qx_cnhw) || !a16(vq) || ((uintptr_t)dW_bf16 & 1u)) return DAQ_ERR_INVALID_ARG;
    const size_t need = daq_workspace_bytes(DAQ_OP_CONV_BWD_FILTER, desc);
    if (need == 0) return DAQ_ERR_UNSUPPORTED;
    if (!ws_ok(workspace, workspace_bytes, need)) return DAQ_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    float* out = reinterpret_cast<float*>(dW_bf16);
    if (bwd_filter_lds_supported(*desc))
        return conv_bwd_filter_lds(*desc, qx_cnhw, s_x, vq, s_chan, out, nullptr, workspace, st, nullptr, true);
    if (bwd_filter_mfma_supported(*desc))
        return conv_bwd_filter_mfma(*desc, qx_cnhw, s_x, vq, s_chan, out, nullptr, workspace, st, true);
    if (depthwise_dw_supported(*desc))
        return conv_bwd_filter_depthwise(*desc, qx_cnhw, s_x, vq, s_chan, out, nullptr, workspace, st, true);
    return conv_bwd_filter_generic(*desc, qx_cnhw, s_x, vq, s_chan, out, nullptr, st, true);
}

extern "C" daq_status daq_conv_bwd_data_int8_chan(const daq_conv_desc* desc, const int8_t* vq, const float* s_chan,
                                                  const int8_t* qw_packed, const float* s_w, float* dX, int32_t* acc_out,
                                                  void* workspace, size_t workspace_bytes, void* stream) {
    if (!desc_valid(desc) || !vq || !s_chan || !qw_packed || !s_w || !dX) return DAQ_ERR_INVALID_ARG;
    if (!a16(vq) || !a16(qw_packed) || !a16(dX) || !a16(acc_out)) return DAQ_ERR_INVALID_ARG;
    const size_t need = daq_workspace_bytes(DAQ_OP_CONV_BWD_DATA, desc);
    if (need == 0) return DAQ_ERR_UNSUPPORTED;
    if (!ws_ok(workspace, workspace_bytes, need)) return DAQ_ERR_WORKSPACE;
    // only where a channel of the data gradient depends on one channel of dY: groups = Cin = Cout
    if (!is_depthwise(*desc) || !depthwise_dx_supported(*desc)) return DAQ_ERR_UNSUPPORTED;
    return conv_bwd_data_depthwise(*desc, vq, s_chan, qw_packed, s_w, dX, acc_out, (hipStream_t)stream, true);
}
