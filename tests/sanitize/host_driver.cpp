// Exercises the host-side logic of libdaq - descriptor validation, int8 layouts, workspace sizes, argument checks of every
// entry point - in a build whose host code is compiled with -fsanitize=address,undefined (tests/test_sanitizers.py).
// No kernel is launched and no GPU is needed: every call below must return before its first launch.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "daq.h"

static int fails = 0;
#define EXPECT(cond)                                                        \
    do {                                                                    \
        if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); ++fails; } \
    } while (0)

int main() {
    std::vector<daq_conv_desc> descs = {
        {2, 3, 9, 7, 5, 3, 3, 1, 1, 1, 1, 1, 1, 1},        {2, 4, 9, 8, 6, 3, 3, 2, 2, 1, 1, 1, 1, 1},
        {1, 3, 15, 15, 4, 7, 7, 2, 2, 3, 3, 1, 1, 1},      {3, 8, 5, 5, 8, 1, 1, 1, 1, 0, 0, 1, 1, 1},
        {2, 6, 7, 7, 6, 3, 3, 1, 1, 1, 1, 1, 1, 6},        {1, 2, 8, 8, 2, 3, 3, 1, 1, 2, 2, 2, 2, 1},
        {64, 64, 56, 56, 256, 1, 1, 1, 1, 0, 0, 1, 1, 1},  {64, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3, 1, 1, 1},
        {128, 96, 112, 112, 96, 3, 3, 2, 2, 1, 1, 1, 1, 96}, {64, 512, 7, 7, 2048, 1, 1, 1, 1, 0, 0, 1, 1, 1},
        {1, 1, 1, 1, 1, 1, 1, 1, 1, 0, 0, 1, 1, 1},        {1, 70000, 1, 1, 70000, 1, 1, 1, 1, 0, 0, 1, 1, 1},
        {4096, 512, 64, 64, 512, 3, 3, 1, 1, 1, 1, 1, 1, 1},   // more than 2^31 elements: unsupported, not a crash
    };
    std::vector<daq_conv_desc> bad = {
        {0, 3, 9, 7, 5, 3, 3, 1, 1, 1, 1, 1, 1, 1}, {2, 3, 9, 7, 5, 3, 3, 0, 1, 1, 1, 1, 1, 1}, {2, 3, 2, 2, 5, 5, 5, 1, 1, 0, 0, 1, 1, 1},
        {2, 4, 9, 7, 6, 3, 3, 1, 1, 1, 1, 1, 1, 4}, {2, 3, 9, 7, 5, 3, 3, 1, 1, -1, 1, 1, 1, 1}, {2, 3, 9, 7, 5, 3, 3, 1, 1, 1, 1, 0, 1, 1},
    };
    for (const auto& d : descs) {
        daq_layout L;
        daq_wpack_layout Lw;
        const daq_status a = daq_layout_vq(&d, &L);
        EXPECT(a == DAQ_OK || a == DAQ_ERR_UNSUPPORTED);
        if (a == DAQ_OK) {
            EXPECT(L.bytes > 0 && L.chan_pitch * L.C == L.bytes);
            EXPECT(daq_layout_qg(&d, &L) == DAQ_OK && daq_layout_qx_nhwc(&d, &L) == DAQ_OK && daq_layout_qx_cnhw(&d, &L) == DAQ_OK);
            EXPECT(daq_layout_qw(&d, &Lw) == DAQ_OK && Lw.bytes >= Lw.off_bwd);
            for (int op = 0; op <= 5; ++op) EXPECT(daq_workspace_bytes((daq_op)op, &d) > 0);
        } else {
            for (int op = 0; op <= 5; ++op) EXPECT(daq_workspace_bytes((daq_op)op, &d) == 0);
        }
        EXPECT(daq_workspace_bytes((daq_op)7, &d) == 0);   // not an operation (inside the range a C++ enum of six values can hold)
        EXPECT(daq_out_h(&d) > 0 && daq_out_w(&d) > 0);
    }
    for (const auto& d : bad) {
        daq_layout L;
        daq_wpack_layout Lw;
        EXPECT(daq_layout_vq(&d, &L) == DAQ_ERR_INVALID_ARG && daq_layout_qw(&d, &Lw) == DAQ_ERR_INVALID_ARG);
        EXPECT(daq_workspace_bytes(DAQ_OP_QUANTIZE_GRAD, &d) == 0);
    }
    EXPECT(daq_layout_vq(nullptr, nullptr) == DAQ_ERR_INVALID_ARG && daq_out_h(nullptr) == 0);
    for (int s = 0; s < 8; ++s) EXPECT(std::strlen(daq_status_string((daq_status)s)) > 0);

    // argument checks of the entry points: null pointers, misaligned pointers (never dereferenced on the host), small workspaces
    const daq_conv_desc d = descs[0];
    float* f = reinterpret_cast<float*>(0x10000);
    int8_t* b = reinterpret_cast<int8_t*>(0x20000);
    uint8_t* u = reinterpret_cast<uint8_t*>(0x30000);
    void* ws = reinterpret_cast<void*>(0x40000);
    EXPECT(daq_quantize_grad(&d, nullptr, f, 1, 0.8f, 0.3f, DAQ_ROUND_NEAREST, 0, b, b, f, f, u, nullptr, ws, 1 << 20, nullptr) == DAQ_ERR_INVALID_ARG);
    EXPECT(daq_quantize_grad(&d, f, f, 1, 0.8f, 0.3f, DAQ_ROUND_NEAREST, 0, b + 1, b, f, f, u, nullptr, ws, 1 << 20, nullptr) == DAQ_ERR_INVALID_ARG);
    EXPECT(daq_quantize_grad(&d, f, f, 1, 0.8f, 0.3f, DAQ_ROUND_NEAREST, 0, b, b, f, f, u, nullptr, ws, 16, nullptr) == DAQ_ERR_WORKSPACE);
    EXPECT(daq_quantize_grad(&d, f, f, 1, 0.8f, 0.3f, DAQ_ROUND_NEAREST, 0, b, b, f, f, u, nullptr, nullptr, 1 << 20, nullptr) == DAQ_ERR_WORKSPACE);
    daq_quantize_opts o = {9, 0, 0, 0};
    EXPECT(daq_quantize_grad_ex(&d, f, f, 1, 0.8f, 0.3f, DAQ_ROUND_NEAREST, 0, &o, b, b, f, f, u, nullptr, ws, 1 << 20, nullptr) == DAQ_ERR_INVALID_ARG);
    o = {0, 9, 0, 0};
    EXPECT(daq_quantize_grad_ex(&d, f, f, 1, 0.8f, 0.3f, DAQ_ROUND_NEAREST, 0, &o, b, b, f, f, u, nullptr, ws, 1 << 20, nullptr) == DAQ_ERR_INVALID_ARG);
    const daq_conv_desc wide = {8, 512, 112, 112, 8192, 1, 1, 1, 1, 0, 0, 1, 1, 1};   // partial results beyond the static array
    EXPECT(daq_workspace_bytes(DAQ_OP_QUANTIZE_GRAD, &wide) > (size_t)DAQ_STATIC_SCRATCH_BYTES);
    EXPECT(daq_quantize_grad_noalloc(&wide, f, f, 1, 0.8f, 0.3f, DAQ_ROUND_NEAREST, 0, b, b, f, f, u, nullptr, nullptr) == DAQ_ERR_SCRATCH_LIMIT);
    EXPECT(daq_conv_fwd_int8(&d, f, nullptr, b, b, b, f, f, f, nullptr, ws, 1 << 20, nullptr) == DAQ_ERR_INVALID_ARG);
    EXPECT(daq_conv_fwd_int8(&d, f, f, b, b, b, f, f, f + 1, nullptr, ws, 1 << 20, nullptr) == DAQ_ERR_INVALID_ARG);
    EXPECT(daq_conv_bwd_data_int8(&d, b, f, b, f, nullptr, nullptr, ws, 1 << 20, nullptr) == DAQ_ERR_INVALID_ARG);
    EXPECT(daq_conv_bwd_data_int8(&d, b, f, b, f, f, nullptr, ws, 0, nullptr) == DAQ_ERR_WORKSPACE);
    EXPECT(daq_conv_bwd_filter_int8(&d, b, f, b, f, nullptr, nullptr, ws, 1 << 20, nullptr) == DAQ_ERR_INVALID_ARG);
    EXPECT(daq_conv_bwd_filter_int8(&d, b, f, b, f, f, nullptr, (char*)ws + 8, 1 << 20, nullptr) == DAQ_ERR_WORKSPACE);
    EXPECT(daq_conv_bwd_int8(&d, b, f, b, f, f, nullptr, b, f, b, nullptr, f, nullptr, ws, 1 << 20, nullptr) == DAQ_ERR_INVALID_ARG);
    EXPECT(daq_conv_bwd_data_int8_bf16(&d, b, f, b, f, nullptr, ws, 1 << 20, nullptr) == DAQ_ERR_INVALID_ARG);
    EXPECT(daq_conv_bwd_filter_int8_bf16(&d, b, f, b, f, nullptr, ws, 1 << 20, nullptr) == DAQ_ERR_INVALID_ARG);
    EXPECT(daq_conv_bwd_data_int8_chan(&d, b, f, b, f, f, nullptr, ws, 1 << 20, nullptr) == DAQ_ERR_UNSUPPORTED);   // not a depthwise layer
    EXPECT(daq_clip_search(&d, f, 1.0f, 0, nullptr, f, reinterpret_cast<int32_t*>(f), ws, 1 << 20, nullptr) == DAQ_ERR_INVALID_ARG);
    EXPECT(daq_clip_search(&d, f, -1.0f, 8, nullptr, f, reinterpret_cast<int32_t*>(f), ws, 1 << 20, nullptr) == DAQ_ERR_INVALID_ARG);
    EXPECT(daq_prof_end(nullptr, 0, nullptr) == DAQ_ERR_INVALID_ARG);

    // 3-D descriptors: carriers, sizes, argument checks
    const daq_conv3d_desc v = {2, 8, 6, 10, 9, 12, 3, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1};
    const daq_conv3d_desc t = {2, 16, 8, 7, 6, 24, 3, 1, 1, 1, 1, 1, 1, 0, 0, 1, 1, 1, 1};
    const daq_conv3d_desc w = {2, 16, 2, 7, 6, 24, 5, 1, 1, 1, 1, 1, 0, 0, 0, 1, 1, 1, 1};   // deeper filter than volume
    daq_conv_desc cx, cg;
    EXPECT(daq_conv3d_carriers(&v, &cx, &cg) == 0 && cx.Hin == 60 && cg.Hin == daq_conv3d_out_d(&v) * daq_conv3d_out_h(&v));
    EXPECT(daq_conv3d_carriers(&t, &cx, &cg) == 1 && cx.kH == 3 && cx.Win == 42);
    EXPECT(daq_conv3d_carriers(&w, &cx, &cg) == -1 && daq_conv3d_carriers(nullptr, &cx, &cg) == -1);
    EXPECT(daq_conv3d_qw_bytes(&v) >= 12 * 8 * 27 && daq_conv3d_qw_bytes(&w) == 0);
    for (int op = 0; op <= 3; ++op) EXPECT(daq_conv3d_workspace_bytes((daq_op)op, &v) > 0 && daq_conv3d_workspace_bytes((daq_op)op, &t) > 0);
    EXPECT(daq_conv3d_fwd_int8(&v, f, nullptr, b, b, b, f, f, f, nullptr, ws, 1 << 20, nullptr) == DAQ_ERR_INVALID_ARG);
    EXPECT(daq_conv3d_fwd_int8(&w, f, f, b, b, b, f, f, f, nullptr, ws, 1 << 20, nullptr) == DAQ_ERR_INVALID_ARG);
    EXPECT(daq_conv3d_bwd_data_int8(&v, b, f, b, f, nullptr, nullptr, ws, 1 << 20, nullptr) == DAQ_ERR_INVALID_ARG);
    EXPECT(daq_conv3d_bwd_filter_int8(&v, b, f, b, f, f, nullptr, nullptr, 1 << 20, nullptr) == DAQ_ERR_WORKSPACE);
    EXPECT(daq_quantize_grad3d(&w, f, f, 1, 0.8f, 0.3f, DAQ_ROUND_NEAREST, 0, nullptr, b, b, f, f, u, nullptr, ws, 1 << 20, nullptr) == DAQ_ERR_INVALID_ARG);

    std::printf(fails ? "host sanitizer run FAILED (%d)\n" : "host sanitizer run ok (%d failures)\n", fails);
    return fails ? 1 : 0;
}
