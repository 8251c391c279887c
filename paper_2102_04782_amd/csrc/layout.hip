// Host-side logic: descriptor validation, int8 buffer layouts, workspace sizes.
// No GPU call is made from this file.
#include <algorithm>

#include "daq_internal.h"

namespace daq {

static int out_dim(int in, int pad, int dil, int k, int stride) {
    const int64_t span = (int64_t)in + 2 * (int64_t)pad - ((int64_t)dil * (k - 1) + 1);
    if (span < 0) return 0;
    return (int)(span / stride + 1);
}

bool desc_valid(const daq_conv_desc* d) {
    if (!d) return false;
    if (d->N <= 0 || d->Cin <= 0 || d->Hin <= 0 || d->Win <= 0 || d->Cout <= 0) return false;
    if (d->kH <= 0 || d->kW <= 0 || d->strideH <= 0 || d->strideW <= 0) return false;
    if (d->padH < 0 || d->padW < 0 || d->dilH <= 0 || d->dilW <= 0 || d->groups <= 0) return false;
    if (d->Cin % d->groups || d->Cout % d->groups) return false;
    if (out_dim(d->Hin, d->padH, d->dilH, d->kH, d->strideH) <= 0) return false;
    if (out_dim(d->Win, d->padW, d->dilW, d->kW, d->strideW) <= 0) return false;
    return true;
}

// Every tensor must be addressable with 31-bit element indices (kernels use 32-bit index math
// inside a channel / image and 64-bit only for base offsets).
static bool sizes_ok(const daq_conv_desc& d) {
    const int64_t lim = (int64_t)1 << 31;
    const int64_t Ho = daq_out_h(&d), Wo = daq_out_w(&d);
    const int64_t ex = (int64_t)d.N * d.Cin * d.Hin * d.Win;
    const int64_t ey = (int64_t)d.N * d.Cout * Ho * Wo;
    const int64_t ew = (int64_t)d.Cout * (d.Cin / d.groups) * d.kH * d.kW;
    const int64_t padded = (int64_t)d.N * (d.Hin + 2 * d.padH + 1) * (d.Win + 2 * d.padW + 1);
    return ex < lim && ey < lim && ew < lim && padded * 16 < lim * 8;
}

// Slot geometry shared by q(X') and vq(G'): both use the same rows-per-image and row pitch so that a
// filter tap is a constant byte offset between the two flattened (n, row, col) axes.
struct Slot {
    int img_rows, row_pitch, phases_h, phases_w, org_h, org_w;
    int64_t lead;   // distance from a gradient position to the activation position of tap (0, 0)
    int64_t halo;   // zero bytes in front of and behind the images of every plane, gradient and activation alike
    int64_t klen;   // bytes of a gradient plane: halo + images + halo, padded to kKAlign
};

static Slot slot_of(const daq_conv_desc& d) {
    Slot s{};
    const int Ho = daq_out_h(&d), Wo = daq_out_w(&d);
    if (d.strideH == 1 && d.strideW == 1) {
        // Unit stride: padding rows/columns are shared between neighbouring rows and images.
        s.phases_h = s.phases_w = 1;
        s.org_h = s.org_w = 0;
        s.row_pitch = d.Win + d.padW > Wo ? d.Win + d.padW : Wo;
        s.img_rows = d.Hin + d.padH > Ho ? d.Hin + d.padH : Ho;
        s.lead = (int64_t)d.padH * s.row_pitch + d.padW;
    } else {
        // Strided: explicit padded coordinates, one plane per stride phase.
        s.phases_h = d.strideH;
        s.phases_w = d.strideW;
        s.org_h = d.padH;
        s.org_w = d.padW;
        const int rp = (int)ceil_div(d.Hin + 2 * d.padH, d.strideH);
        const int cp = (int)ceil_div(d.Win + 2 * d.padW, d.strideW);
        s.img_rows = rp > Ho ? rp : Ho;
        s.row_pitch = cp > Wo ? cp : Wo;
        s.lead = 0;
    }
    // Every neighbour a filter tap can reach from a real element, in either direction, is an addressable zero:
    // kernels that walk a plane with shifted reads (filter gradient, depthwise data gradient) need no bounds tests.
    s.halo = round_up((int64_t)((d.kH - 1) * d.dilH + 1) * s.row_pitch + (int64_t)(d.kW - 1) * d.dilW + 16, 64);
    s.klen = round_up(2 * s.halo + (int64_t)d.N * s.img_rows * s.row_pitch, kKAlign);
    return s;
}

static void fill_cnhw(daq_layout* L, const Slot& s, int C, int N, int H, int W, bool activation,
                      const daq_conv_desc& d) {
    L->kind = DAQ_LAYOUT_CNHW;
    L->C = C; L->N = N; L->H = H; L->W = W;
    L->c_pitch = 0;
    L->img_rows = s.img_rows;
    L->row_pitch = s.row_pitch;
    if (activation) {
        L->phases_h = s.phases_h; L->phases_w = s.phases_w;
        L->org_h = s.org_h; L->org_w = s.org_w;
        L->lead = s.halo + s.lead;
        // a tap reads up to (kH-1)*dilH rows and (kW-1)*dilW columns past the gradient's position
        const int64_t reach = (int64_t)((d.kH - 1) * d.dilH / d.strideH + 1) * s.row_pitch +
                              (int64_t)(d.kW - 1) * d.dilW / d.strideW + 64;
        L->plane_pitch = round_up(s.lead + s.klen + reach, kKAlign);
        L->chan_pitch = L->plane_pitch * s.phases_h * s.phases_w;
    } else {
        L->phases_h = L->phases_w = 1;
        L->org_h = L->org_w = 0;
        L->lead = s.halo;
        L->plane_pitch = s.klen;
        L->chan_pitch = s.klen;
    }
    L->bytes = L->chan_pitch * C;
}

static void fill_nhwc(daq_layout* L, int C, int N, int H, int W) {
    L->kind = DAQ_LAYOUT_NHWC;
    L->C = C; L->N = N; L->H = H; L->W = W;
    L->c_pitch = (int32_t)round_up(C, 16);
    L->img_rows = L->row_pitch = 0;
    L->phases_h = L->phases_w = 1;
    L->org_h = L->org_w = 0;
    L->chan_pitch = L->plane_pitch = L->lead = 0;
    L->bytes = round_up((int64_t)N * H * W * L->c_pitch, 256);
}

}  // namespace daq

using namespace daq;

extern "C" {

int32_t daq_out_h(const daq_conv_desc* d) {
    return d ? out_dim(d->Hin, d->padH, d->dilH, d->kH, d->strideH) : 0;
}
int32_t daq_out_w(const daq_conv_desc* d) {
    return d ? out_dim(d->Win, d->padW, d->dilW, d->kW, d->strideW) : 0;
}

daq_status daq_layout_vq(const daq_conv_desc* d, daq_layout* out) {
    if (!desc_valid(d) || !out) return DAQ_ERR_INVALID_ARG;
    if (!sizes_ok(*d)) return DAQ_ERR_UNSUPPORTED;
    fill_cnhw(out, slot_of(*d), d->Cout, d->N, daq_out_h(d), daq_out_w(d), false, *d);
    return DAQ_OK;
}

daq_status daq_layout_qg(const daq_conv_desc* d, daq_layout* out) {
    if (!desc_valid(d) || !out) return DAQ_ERR_INVALID_ARG;
    if (!sizes_ok(*d)) return DAQ_ERR_UNSUPPORTED;
    if (is_depthwise(*d))
        fill_cnhw(out, slot_of(*d), d->Cout, d->N, daq_out_h(d), daq_out_w(d), false, *d);
    else
        fill_nhwc(out, d->Cout, d->N, daq_out_h(d), daq_out_w(d));
    return DAQ_OK;
}

daq_status daq_layout_qx_nhwc(const daq_conv_desc* d, daq_layout* out) {
    if (!desc_valid(d) || !out) return DAQ_ERR_INVALID_ARG;
    if (!sizes_ok(*d)) return DAQ_ERR_UNSUPPORTED;
    fill_nhwc(out, d->Cin, d->N, d->Hin, d->Win);
    return DAQ_OK;
}

daq_status daq_layout_qx_cnhw(const daq_conv_desc* d, daq_layout* out) {
    if (!desc_valid(d) || !out) return DAQ_ERR_INVALID_ARG;
    if (!sizes_ok(*d)) return DAQ_ERR_UNSUPPORTED;
    fill_cnhw(out, slot_of(*d), d->Cin, d->N, d->Hin, d->Win, true, *d);
    return DAQ_OK;
}

daq_status daq_layout_qw(const daq_conv_desc* d, daq_wpack_layout* out) {
    if (!desc_valid(d) || !out) return DAQ_ERR_INVALID_ARG;
    if (!sizes_ok(*d)) return DAQ_ERR_UNSUPPORTED;
    const int cig = d->Cin / d->groups, cog = d->Cout / d->groups;
    const int64_t taps = (int64_t)d->kH * d->kW;
    out->cig_pitch = (int32_t)round_up(cig, 16);
    out->cog_pitch = (int32_t)round_up(cog, 16);
    out->off_plain = 0;
    out->off_fwd = round_up((int64_t)d->Cout * cig * taps, 256);
    out->off_bwd = out->off_fwd + round_up(taps * d->Cout * out->cig_pitch, 256);
    out->bytes = out->off_bwd + round_up(taps * d->Cin * out->cog_pitch, 256);
    out->off_fwd_frag = out->off_bwd_frag = out->bytes;
    if (d->groups == 1) {
        out->off_bwd_frag = out->off_fwd_frag + ceil_div(d->Cin, 64) * taps * ceil_div(d->Cout, 32) * 2048;
        out->bytes = out->off_bwd_frag + ceil_div(d->Cout, 64) * taps * ceil_div(d->Cin, 32) * 2048;
    }
    return DAQ_OK;
}

size_t daq_workspace_bytes(daq_op op, const daq_conv_desc* d) {
    if (!desc_valid(d) || !sizes_ok(*d)) return 0;
    switch (op) {
        case DAQ_OP_QUANTIZE_GRAD: return quantize_grad_ws_bytes(*d);
        case DAQ_OP_CONV_FWD: return fwd_quant_ws_bytes(*d);
        case DAQ_OP_CONV_BWD_DATA: return 256;
        case DAQ_OP_CONV_BWD_FILTER: return 256 + std::max({bwd_filter_mfma_ws_bytes(*d), bwd_filter_lds_ws_bytes(*d), depthwise_dw_ws_bytes(*d)});
        case DAQ_OP_CONV_BWD: return daq_workspace_bytes(DAQ_OP_CONV_BWD_FILTER, d) + daq_workspace_bytes(DAQ_OP_CONV_BWD_DATA, d);
        case DAQ_OP_CLIP_SEARCH: return clip_search_ws_bytes(*d);
        default: return 0;
    }
}

const char* daq_status_string(daq_status s) {
    switch (s) {
        case DAQ_OK: return "ok";
        case DAQ_ERR_INVALID_ARG: return "invalid argument";
        case DAQ_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case DAQ_ERR_UNSUPPORTED: return "unsupported problem size";
        case DAQ_ERR_HIP: return "HIP error";
        case DAQ_ERR_SCRATCH_LIMIT: return "problem needs more scratch than the library's static buffer holds";
        default: return "unknown status";
    }
}

}  // extern "C"
