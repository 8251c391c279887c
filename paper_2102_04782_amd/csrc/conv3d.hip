// 3-D convolution layers (the video-classification experiment: the depth axis is treated like height and width).
//
// Where the 3-D problem IS a 2-D problem - a filter that does not extend in height and width (time-only filters and
// pointwise layers: depth becomes the row axis and a whole frame the column axis), or a volume of depth one - the entry
// points hand it to the 2-D entry points, matrix-core kernels included; the views involved are pure reinterpretations of
// the NCDHW tensors.  Every other layer (3 x 3 x 3 and friends) runs on the direct integer kernels below: exact, not fast.
//
// The int8 tensors of a 3-D layer use the 2-D layouts of two "carrier" problems (daq_conv3d_carriers): the activation
// side sees (N, Cin, Din*Hin, Win), the gradient side (N, Cout, Do*Ho, Wo), so that the 2-D quantizers serve unchanged -
// the statistics of Algorithm 1 run over all of (n, d, h, w) either way.
#include <algorithm>

#include "daq_internal.h"

namespace daq {

namespace {

constexpr int kBlock = 256;

int out_dim3(int in, int pad, int dil, int k, int stride) {
    const int64_t span = (int64_t)in + 2 * (int64_t)pad - ((int64_t)dil * (k - 1) + 1);
    return span < 0 ? 0 : (int)(span / stride + 1);
}

struct Geo3 {
    int N, Cin, Din, Hin, Win, Cout, kD, kH, kW, sD, sH, sW, pD, pH, pW, dD, dH, dW, groups, Do, Ho, Wo, cig, cog;
};

bool desc3_valid(const daq_conv3d_desc* d) {
    if (!d) return false;
    if (d->N <= 0 || d->Cin <= 0 || d->Din <= 0 || d->Hin <= 0 || d->Win <= 0 || d->Cout <= 0) return false;
    if (d->kD <= 0 || d->kH <= 0 || d->kW <= 0 || d->strideD <= 0 || d->strideH <= 0 || d->strideW <= 0) return false;
    if (d->padD < 0 || d->padH < 0 || d->padW < 0 || d->dilD <= 0 || d->dilH <= 0 || d->dilW <= 0 || d->groups <= 0) return false;
    if (d->Cin % d->groups || d->Cout % d->groups) return false;
    if (out_dim3(d->Din, d->padD, d->dilD, d->kD, d->strideD) <= 0) return false;
    if (out_dim3(d->Hin, d->padH, d->dilH, d->kH, d->strideH) <= 0) return false;
    if (out_dim3(d->Win, d->padW, d->dilW, d->kW, d->strideW) <= 0) return false;
    // the carriers fold depth into the row axis
    if ((int64_t)d->Din * d->Hin >= ((int64_t)1 << 30)) return false;
    return true;
}

Geo3 geo3_of(const daq_conv3d_desc& d) {
    return Geo3{d.N, d.Cin, d.Din, d.Hin, d.Win, d.Cout, d.kD, d.kH, d.kW, d.strideD, d.strideH, d.strideW, d.padD, d.padH, d.padW,
                d.dilD, d.dilH, d.dilW, d.groups, out_dim3(d.Din, d.padD, d.dilD, d.kD, d.strideD),
                out_dim3(d.Hin, d.padH, d.dilH, d.kH, d.strideH), out_dim3(d.Win, d.padW, d.dilW, d.kW, d.strideW),
                d.Cin / d.groups, d.Cout / d.groups};
}

daq_conv_desc plain2d(int N, int Cin, int H, int W, int Cout, int groups) {
    return daq_conv_desc{N, Cin, H, W, Cout, 1, 1, 1, 1, 0, 0, 1, 1, groups};
}

// 1: *fold computes the layer exactly on reinterpreted tensors; 0: no such 2-D problem.
int fold_of(const daq_conv3d_desc& d, daq_conv_desc* fold) {
    if (d.kH == 1 && d.kW == 1 && d.strideH == 1 && d.strideW == 1 && d.padH == 0 && d.padW == 0 &&
        (int64_t)d.Hin * d.Win < ((int64_t)1 << 30)) {
        // the filter extends in depth only: rows = depth, columns = a whole frame
        *fold = daq_conv_desc{d.N, d.Cin, d.Din, d.Hin * d.Win, d.Cout, d.kD, 1, d.strideD, 1, d.padD, 0, d.dilD, 1, d.groups};
        return 1;
    }
    if (d.Din == 1 && d.kD == 1 && d.padD == 0) {   // a volume of depth one is an image
        *fold = daq_conv_desc{d.N, d.Cin, d.Hin, d.Win, d.Cout, d.kH, d.kW, d.strideH, d.strideW, d.padH, d.padW, d.dilH, d.dilW, d.groups};
        return 1;
    }
    return 0;
}

__device__ __forceinline__ float dq2(int32_t acc, float sa, float sb) { return (float)acc * ((sa / 127.0f) * (sb / 127.0f)); }

// Y[n,co,od,ho,wo]: X from the NHWC carrier (rows = depth*Hin + h, channels innermost), W from the plain filter.
__global__ __launch_bounds__(kBlock) void k3_fwd(Geo3 g, NhwcView X, const int8_t* __restrict__ qx, const int8_t* __restrict__ qw,
                                                 const float* s_x, const float* s_w, float* __restrict__ Y,
                                                 int32_t* __restrict__ acc_out) {
    const int64_t total = (int64_t)g.N * g.Cout * g.Do * g.Ho * g.Wo;
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    const int64_t at = i;
    const int wo = (int)(i % g.Wo); i /= g.Wo;
    const int ho = (int)(i % g.Ho); i /= g.Ho;
    const int od = (int)(i % g.Do); i /= g.Do;
    const int co = (int)(i % g.Cout);
    const int n = (int)(i / g.Cout);
    const int grp = co / g.cog;
    const int taps = g.kD * g.kH * g.kW;
    int32_t a = 0;
    for (int kd = 0; kd < g.kD; ++kd) {
        const int z = od * g.sD + kd * g.dD - g.pD;
        if (z < 0 || z >= g.Din) continue;
        for (int kh = 0; kh < g.kH; ++kh) {
            const int h = ho * g.sH + kh * g.dH - g.pH;
            if (h < 0 || h >= g.Hin) continue;
            for (int kw = 0; kw < g.kW; ++kw) {
                const int w = wo * g.sW + kw * g.dW - g.pW;
                if (w < 0 || w >= g.Win) continue;
                const int8_t* xp = qx + X.offset(n, grp * g.cig, z * g.Hin + h, w);
                const int8_t* wp = qw + (int64_t)co * g.cig * taps + (kd * g.kH + kh) * g.kW + kw;
                for (int cl = 0; cl < g.cig; ++cl) a += (int32_t)xp[cl] * (int32_t)wp[(int64_t)cl * taps];
            }
        }
    }
    Y[at] = dq2(a, *s_x, *s_w);
    if (acc_out) acc_out[at] = a;
}

// dX[n,ci,z,h,w]: G from the NHWC carrier of the gradient (rows = od*Ho + ho).
__global__ __launch_bounds__(kBlock) void k3_bwd_data(Geo3 g, NhwcView G, const int8_t* __restrict__ qg, const int8_t* __restrict__ qw,
                                                      const float* s_g, const float* s_w, float* __restrict__ dX,
                                                      int32_t* __restrict__ acc_out) {
    const int64_t total = (int64_t)g.N * g.Cin * g.Din * g.Hin * g.Win;
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    const int64_t at = i;
    const int w = (int)(i % g.Win); i /= g.Win;
    const int h = (int)(i % g.Hin); i /= g.Hin;
    const int z = (int)(i % g.Din); i /= g.Din;
    const int ci = (int)(i % g.Cin);
    const int n = (int)(i / g.Cin);
    const int grp = ci / g.cig, cl = ci % g.cig;
    const int taps = g.kD * g.kH * g.kW;
    int32_t a = 0;
    for (int kd = 0; kd < g.kD; ++kd) {
        const int zn = z + g.pD - kd * g.dD;
        if (zn < 0 || zn % g.sD || zn / g.sD >= g.Do) continue;
        for (int kh = 0; kh < g.kH; ++kh) {
            const int hn = h + g.pH - kh * g.dH;
            if (hn < 0 || hn % g.sH || hn / g.sH >= g.Ho) continue;
            for (int kw = 0; kw < g.kW; ++kw) {
                const int wn = w + g.pW - kw * g.dW;
                if (wn < 0 || wn % g.sW || wn / g.sW >= g.Wo) continue;
                const int8_t* gp = qg + G.offset(n, grp * g.cog, (zn / g.sD) * g.Ho + hn / g.sH, wn / g.sW);
                const int8_t* wp = qw + ((int64_t)grp * g.cog * g.cig + cl) * taps + (kd * g.kH + kh) * g.kW + kw;
                for (int col = 0; col < g.cog; ++col) a += (int32_t)gp[col] * (int32_t)wp[(int64_t)col * g.cig * taps];
            }
        }
    }
    dX[at] = dq2(a, *s_w, *s_g);
    if (acc_out) acc_out[at] = a;
}

// dW[co,cl,kd,kh,kw]: one workgroup per filter element, threads stride over (n, od, ho, wo); both operands channel-major.
__global__ __launch_bounds__(kBlock) void k3_bwd_filter(Geo3 g, CnhwView X, CnhwView G, const int8_t* __restrict__ qx,
                                                        const int8_t* __restrict__ vq, const float* s_x,
                                                        const float* __restrict__ s_chan, float* __restrict__ dW,
                                                        int32_t* __restrict__ acc_out) {
    int64_t e = blockIdx.x;
    const int64_t at = e;
    const int kw = (int)(e % g.kW); e /= g.kW;
    const int kh = (int)(e % g.kH); e /= g.kH;
    const int kd = (int)(e % g.kD); e /= g.kD;
    const int cl = (int)(e % g.cig);
    const int co = (int)(e / g.cig);
    const int ci = (co / g.cog) * g.cig + cl;
    const int HWo = g.Ho * g.Wo;
    const int64_t vol = (int64_t)g.Do * HWo, K = (int64_t)g.N * vol;
    int32_t a = 0;
    for (int64_t m = threadIdx.x; m < K; m += kBlock) {
        const int n = (int)(m / vol);
        const int64_t r = m - (int64_t)n * vol;
        const int od = (int)(r / HWo);
        const int r2 = (int)(r - (int64_t)od * HWo);
        const int ho = r2 / g.Wo, wo = r2 - ho * g.Wo;
        const int z = od * g.sD + kd * g.dD - g.pD, h = ho * g.sH + kh * g.dH - g.pH, w = wo * g.sW + kw * g.dW - g.pW;
        if (z < 0 || z >= g.Din || h < 0 || h >= g.Hin || w < 0 || w >= g.Win) continue;
        a += (int32_t)qx[X.offset(n, ci, z * g.Hin + h, w)] * (int32_t)vq[G.offset(n, co, od * g.Ho + ho, wo)];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) a += __shfl_down(a, o);
    __shared__ int32_t part[kBlock / kWave];
    if (threadIdx.x % kWave == 0) part[threadIdx.x / kWave] = a;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kBlock / kWave; ++w) a += part[w];
        dW[at] = dq2(a, *s_x, s_chan[co]);
        if (acc_out) acc_out[at] = a;
    }
}

// max |w| of the filter, then its codes in the plain arrangement [Cout][Cin/groups][kD][kH][kW]
__global__ __launch_bounds__(kBlock) void k3_absmax(const float* __restrict__ x, int64_t n, uint32_t* bits) {
    float m = 0.0f;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock) m = fmaxf(m, fabsf(x[i]));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_down(m, o));
    if (threadIdx.x % kWave == 0) atomicMax(bits, __float_as_uint(m));   // bit patterns of non-negative floats order like the floats
}
__global__ void k3_zero(uint32_t* p) { *p = 0u; }
__global__ __launch_bounds__(kBlock) void k3_quant_plain(const float* __restrict__ W, int64_t n, const uint32_t* bits, float* s_w,
                                                         int8_t* __restrict__ out, int64_t out_bytes) {
    const float v = __uint_as_float(*bits);
    const float s = (v >= kTinyScale) ? v : 0.0f;
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i == 0) *s_w = s;
    if (i >= out_bytes) return;
    const float inv = (s >= kTinyScale) ? 127.0f / s : 0.0f;
    out[i] = i < n ? (int8_t)(int)rintf(fminf(fmaxf(W[i] * inv, -127.0f), 127.0f)) : (int8_t)0;
}

int64_t elems_w(const daq_conv3d_desc& d) { return (int64_t)d.Cout * (d.Cin / d.groups) * d.kD * d.kH * d.kW; }

bool sizes3_ok(const daq_conv3d_desc& d) {
    const Geo3 g = geo3_of(d);
    const int64_t lim = (int64_t)1 << 31;
    return (int64_t)g.N * g.Cin * g.Din * g.Hin * g.Win < lim && (int64_t)g.N * g.Cout * g.Do * g.Ho * g.Wo < lim && elems_w(d) < lim &&
           (int64_t)g.Do * g.Ho < ((int64_t)1 << 30);
}

bool ws_ok(const void* ws, size_t have, size_t need) { return ws && have >= need && ((uintptr_t)ws & 255u) == 0; }
bool a16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace
}  // namespace daq

using namespace daq;

extern "C" int32_t daq_conv3d_out_d(const daq_conv3d_desc* d) { return d ? out_dim3(d->Din, d->padD, d->dilD, d->kD, d->strideD) : 0; }
extern "C" int32_t daq_conv3d_out_h(const daq_conv3d_desc* d) { return d ? out_dim3(d->Hin, d->padH, d->dilH, d->kH, d->strideH) : 0; }
extern "C" int32_t daq_conv3d_out_w(const daq_conv3d_desc* d) { return d ? out_dim3(d->Win, d->padW, d->dilW, d->kW, d->strideW) : 0; }

extern "C" int32_t daq_conv3d_carriers(const daq_conv3d_desc* desc, daq_conv_desc* cx, daq_conv_desc* cg) {
    if (!desc3_valid(desc) || !cx || !cg || !sizes3_ok(*desc)) return -1;
    daq_conv_desc fold;
    if (fold_of(*desc, &fold)) {
        *cx = fold;
        *cg = fold;
        return 1;
    }
    const Geo3 g = geo3_of(*desc);
    *cx = plain2d(g.N, g.Cin, g.Din * g.Hin, g.Win, g.Cin, 1);
    *cg = plain2d(g.N, g.Cout, g.Do * g.Ho, g.Wo, g.Cout, 1);
    return 0;
}

extern "C" int64_t daq_conv3d_qw_bytes(const daq_conv3d_desc* desc) {
    daq_conv_desc cx, cg;
    const int kind = daq_conv3d_carriers(desc, &cx, &cg);
    if (kind < 0) return 0;
    if (kind == 1) {
        daq_wpack_layout L;
        return daq_layout_qw(&cx, &L) == DAQ_OK ? L.bytes : 0;
    }
    return round_up(elems_w(*desc), 256);
}

extern "C" size_t daq_conv3d_workspace_bytes(daq_op op, const daq_conv3d_desc* desc) {
    daq_conv_desc cx, cg;
    const int kind = daq_conv3d_carriers(desc, &cx, &cg);
    if (kind < 0) return 0;
    if (kind == 1) return daq_workspace_bytes(op, &cx);
    switch (op) {
        case DAQ_OP_QUANTIZE_GRAD: return daq_workspace_bytes(DAQ_OP_QUANTIZE_GRAD, &cg);
        case DAQ_OP_CONV_FWD: return daq_workspace_bytes(DAQ_OP_CONV_FWD, &cx);
        case DAQ_OP_CONV_BWD_DATA:
        case DAQ_OP_CONV_BWD_FILTER: return 256;
        default: return 0;
    }
}

extern "C" daq_status daq_quantize_grad3d(const daq_conv3d_desc* desc, const void* dY, float* s_state, float k, float A, float lambda,
                                          daq_round mode, uint64_t seed, const daq_quantize_opts* opts, int8_t* vq, int8_t* qg,
                                          float* s_chan, float* s_global, uint8_t* cls, float* stats, void* workspace,
                                          size_t workspace_bytes, void* stream) {
    daq_conv_desc cx, cg;
    const int kind = daq_conv3d_carriers(desc, &cx, &cg);
    if (kind < 0) return desc3_valid(desc) ? DAQ_ERR_UNSUPPORTED : DAQ_ERR_INVALID_ARG;
    return daq_quantize_grad_ex(&cg, dY, s_state, k, A, lambda, mode, seed, opts, vq, qg, s_chan, s_global, cls, stats, workspace,
                                workspace_bytes, stream);
}

extern "C" daq_status daq_conv3d_fwd_int8(const daq_conv3d_desc* desc, const float* X, const float* W, int8_t* qx_nhwc,
                                          int8_t* qx_cnhw, int8_t* qw, float* s_x, float* s_w, float* Y, int32_t* acc_out,
                                          void* workspace, size_t workspace_bytes, void* stream) {
    daq_conv_desc cx, cg;
    const int kind = daq_conv3d_carriers(desc, &cx, &cg);
    if (kind < 0) return desc3_valid(desc) ? DAQ_ERR_UNSUPPORTED : DAQ_ERR_INVALID_ARG;
    if (kind == 1) return daq_conv_fwd_int8(&cx, X, W, qx_nhwc, qx_cnhw, qw, s_x, s_w, Y, acc_out, workspace, workspace_bytes, stream);
    if (!X || !W || !qx_nhwc || !qx_cnhw || !qw || !s_x || !s_w || !Y) return DAQ_ERR_INVALID_ARG;
    if (((uintptr_t)X & 3u) || ((uintptr_t)W & 3u) || !a16(qx_nhwc) || !a16(qx_cnhw) || !a16(qw) || !a16(Y) || !a16(acc_out))
        return DAQ_ERR_INVALID_ARG;
    if (!ws_ok(workspace, workspace_bytes, daq_conv3d_workspace_bytes(DAQ_OP_CONV_FWD, desc))) return DAQ_ERR_WORKSPACE;
    daq_status rc = quantize_activation_check(cx, X);
    if (rc != DAQ_OK) return rc;
    daq_layout Ln;
    if (daq_layout_qx_nhwc(&cx, &Ln) != DAQ_OK) return DAQ_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    rc = quantize_activation(cx, X, qx_nhwc, qx_cnhw, s_x, workspace, st, DAQ_SCHEDULE_AUTO);
    if (rc != DAQ_OK) return rc;
    uint32_t* bits = (uint32_t*)workspace + 32;
    const int64_t nw = elems_w(*desc), wb = round_up(nw, 256);
    DAQ_LAUNCH("fill", st, hipLaunchKernelGGL(k3_zero, dim3(1), dim3(1), 0, st, bits));
    DAQ_LAUNCH("absmax", st, hipLaunchKernelGGL(k3_absmax, dim3((unsigned)std::min<int64_t>(ceil_div(nw, kBlock), 1024)), dim3(kBlock), 0, st, W, nw, bits));
    DAQ_LAUNCH("pack_w", st, hipLaunchKernelGGL(k3_quant_plain, dim3((unsigned)ceil_div(wb, kBlock)), dim3(kBlock), 0, st, W, nw, bits, s_w, qw, wb));
    const Geo3 g = geo3_of(*desc);
    const int64_t total = (int64_t)g.N * g.Cout * g.Do * g.Ho * g.Wo;
    DAQ_LAUNCH("conv3d_fwd_direct", st,
               hipLaunchKernelGGL(k3_fwd, dim3((unsigned)ceil_div(total, kBlock)), dim3(kBlock), 0, st, g, nhwc_view(Ln), qx_nhwc, qw, s_x,
                                  s_w, Y, acc_out));
    return DAQ_OK;
}

extern "C" daq_status daq_conv3d_bwd_data_int8(const daq_conv3d_desc* desc, const int8_t* qg, const float* s_global, const int8_t* qw,
                                               const float* s_w, float* dX, int32_t* acc_out, void* workspace,
                                               size_t workspace_bytes, void* stream) {
    daq_conv_desc cx, cg;
    const int kind = daq_conv3d_carriers(desc, &cx, &cg);
    if (kind < 0) return desc3_valid(desc) ? DAQ_ERR_UNSUPPORTED : DAQ_ERR_INVALID_ARG;
    if (kind == 1) return daq_conv_bwd_data_int8(&cx, qg, s_global, qw, s_w, dX, acc_out, workspace, workspace_bytes, stream);
    if (!qg || !s_global || !qw || !s_w || !dX) return DAQ_ERR_INVALID_ARG;
    if (!a16(qg) || !a16(qw) || !a16(dX) || !a16(acc_out)) return DAQ_ERR_INVALID_ARG;
    if (!ws_ok(workspace, workspace_bytes, 256)) return DAQ_ERR_WORKSPACE;
    daq_layout Lg;
    if (daq_layout_qg(&cg, &Lg) != DAQ_OK || Lg.kind != DAQ_LAYOUT_NHWC) return DAQ_ERR_UNSUPPORTED;
    const Geo3 g = geo3_of(*desc);
    const int64_t total = (int64_t)g.N * g.Cin * g.Din * g.Hin * g.Win;
    hipStream_t st = (hipStream_t)stream;
    DAQ_LAUNCH("conv3d_bwd_data_direct", st,
               hipLaunchKernelGGL(k3_bwd_data, dim3((unsigned)ceil_div(total, kBlock)), dim3(kBlock), 0, st, g, nhwc_view(Lg), qg, qw,
                                  s_global, s_w, dX, acc_out));
    return DAQ_OK;
}

extern "C" daq_status daq_conv3d_bwd_filter_int8(const daq_conv3d_desc* desc, const int8_t* qx_cnhw, const float* s_x, const int8_t* vq,
                                                 const float* s_chan, float* dW, int32_t* acc_out, void* workspace,
                                                 size_t workspace_bytes, void* stream) {
    daq_conv_desc cx, cg;
    const int kind = daq_conv3d_carriers(desc, &cx, &cg);
    if (kind < 0) return desc3_valid(desc) ? DAQ_ERR_UNSUPPORTED : DAQ_ERR_INVALID_ARG;
    if (kind == 1) return daq_conv_bwd_filter_int8(&cx, qx_cnhw, s_x, vq, s_chan, dW, acc_out, workspace, workspace_bytes, stream);
    if (!qx_cnhw || !s_x || !vq || !s_chan || !dW) return DAQ_ERR_INVALID_ARG;
    if (!a16(qx_cnhw) || !a16(vq) || ((uintptr_t)dW & 3u) || ((uintptr_t)acc_out & 3u)) return DAQ_ERR_INVALID_ARG;
    if (!ws_ok(workspace, workspace_bytes, 256)) return DAQ_ERR_WORKSPACE;
    daq_layout Lx, Lg;
    if (daq_layout_qx_cnhw(&cx, &Lx) != DAQ_OK || daq_layout_vq(&cg, &Lg) != DAQ_OK) return DAQ_ERR_UNSUPPORTED;
    const Geo3 g = geo3_of(*desc);
    hipStream_t st = (hipStream_t)stream;
    DAQ_LAUNCH("conv3d_bwd_filter_direct", st,
               hipLaunchKernelGGL(k3_bwd_filter, dim3((unsigned)elems_w(*desc)), dim3(kBlock), 0, st, g, cnhw_view(Lx), cnhw_view(Lg),
                                  qx_cnhw, vq, s_x, s_chan, dW, acc_out));
    return DAQ_OK;
}
