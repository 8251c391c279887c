// Direct int8 convolution kernels for descriptors nothing else covers (grouped layers that are not
// depthwise, filters with more taps than the matrix-core kernels take, depthwise filter gradients with
// more than nine taps, the depthwise forward pass).
// Plain integer ALU work: one thread (or one workgroup) per output element, int32 accumulation,
// de-quantization in the epilogue.  Correct for every valid descriptor.
#include "daq_internal.h"

namespace daq {

namespace {

constexpr int kBlock = 256;

struct Geo {
    int N, Cin, Hin, Win, Cout, kH, kW, sH, sW, pH, pW, dH, dW, groups, Ho, Wo, cig, cog;
};

Geo geo_of(const daq_conv_desc& d) {
    Geo g{d.N, d.Cin, d.Hin, d.Win, d.Cout, d.kH, d.kW, d.strideH, d.strideW, d.padH, d.padW, d.dilH, d.dilW,
          d.groups, daq_out_h(&d), daq_out_w(&d), d.Cin / d.groups, d.Cout / d.groups};
    return g;
}

__device__ __forceinline__ float dq2(int32_t acc, float sa, float sb) {
    return (float)acc * ((sa / 127.0f) * (sb / 127.0f));
}

// Y[n,co,ho,wo]; X read from NHWC, W from the plain copy.
__global__ __launch_bounds__(kBlock) void k_fwd(Geo g, NhwcView X, const int8_t* __restrict__ qx,
                                                const int8_t* __restrict__ qw, const float* s_x, const float* s_w,
                                                float* __restrict__ Y, int32_t* __restrict__ acc_out) {
    const int64_t total = (int64_t)g.N * g.Cout * g.Ho * g.Wo;
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    const int wo = (int)(i % g.Wo);
    const int ho = (int)((i / g.Wo) % g.Ho);
    const int co = (int)((i / ((int64_t)g.Wo * g.Ho)) % g.Cout);
    const int n = (int)(i / ((int64_t)g.Wo * g.Ho * g.Cout));
    const int grp = co / g.cog;
    int32_t a = 0;
    for (int kh = 0; kh < g.kH; ++kh) {
        const int h = ho * g.sH + kh * g.dH - g.pH;
        if (h < 0 || h >= g.Hin) continue;
        for (int kw = 0; kw < g.kW; ++kw) {
            const int w = wo * g.sW + kw * g.dW - g.pW;
            if (w < 0 || w >= g.Win) continue;
            const int8_t* xp = qx + X.offset(n, grp * g.cig, h, w);
            const int8_t* wp = qw + (((int64_t)co * g.cig) * g.kH + kh) * g.kW + kw;
            for (int cl = 0; cl < g.cig; ++cl) a += (int32_t)xp[cl] * (int32_t)wp[(int64_t)cl * g.kH * g.kW];
        }
    }
    Y[i] = dq2(a, *s_x, *s_w);
    if (acc_out) acc_out[i] = a;
}

// dX[n,ci,h,w]; G read through its layout (NHWC, or CNHW for depthwise layers).
template <bool G_NHWC>
__global__ __launch_bounds__(kBlock) void k_bwd_data(Geo g, NhwcView Gn, CnhwView Gc, const int8_t* __restrict__ qg,
                                                     const int8_t* __restrict__ qw, const float* s_g,
                                                     const float* s_w, float* __restrict__ dX,
                                                     int32_t* __restrict__ acc_out, int bf16) {
    const int64_t total = (int64_t)g.N * g.Cin * g.Hin * g.Win;
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    const int w = (int)(i % g.Win);
    const int h = (int)((i / g.Win) % g.Hin);
    const int ci = (int)((i / ((int64_t)g.Win * g.Hin)) % g.Cin);
    const int n = (int)(i / ((int64_t)g.Win * g.Hin * g.Cin));
    const int grp = ci / g.cig, cl = ci % g.cig;
    int32_t a = 0;
    for (int kh = 0; kh < g.kH; ++kh) {
        const int hn = h + g.pH - kh * g.dH;
        if (hn < 0 || hn % g.sH) continue;
        const int ho = hn / g.sH;
        if (ho >= g.Ho) continue;
        for (int kw = 0; kw < g.kW; ++kw) {
            const int wn = w + g.pW - kw * g.dW;
            if (wn < 0 || wn % g.sW) continue;
            const int wo = wn / g.sW;
            if (wo >= g.Wo) continue;
            for (int col = 0; col < g.cog; ++col) {
                const int co = grp * g.cog + col;
                const int8_t gv = G_NHWC ? qg[Gn.offset(n, co, ho, wo)] : qg[Gc.offset(n, co, ho, wo)];
                const int8_t wv = qw[(((int64_t)co * g.cig + cl) * g.kH + kh) * g.kW + kw];
                a += (int32_t)gv * (int32_t)wv;
            }
        }
    }
    store_result(dX, i, dq2(a, *s_w, *s_g), bf16);
    if (acc_out) acc_out[i] = a;
}

// dW[co,cl,kh,kw]: one workgroup per filter element, threads stride over (n, ho, wo).
__global__ __launch_bounds__(kBlock) void k_bwd_filter(Geo g, CnhwView X, CnhwView G, const int8_t* __restrict__ qx,
                                                       const int8_t* __restrict__ vq, const float* s_x,
                                                       const float* __restrict__ s_chan, float* __restrict__ dW,
                                                       int32_t* __restrict__ acc_out, int bf16) {
    const int64_t e = blockIdx.x;
    const int kw = (int)(e % g.kW);
    const int kh = (int)((e / g.kW) % g.kH);
    const int cl = (int)((e / ((int64_t)g.kW * g.kH)) % g.cig);
    const int co = (int)(e / ((int64_t)g.kW * g.kH * g.cig));
    const int ci = (co / g.cog) * g.cig + cl;
    const int HWo = g.Ho * g.Wo;
    const int64_t K = (int64_t)g.N * HWo;
    int32_t a = 0;
    for (int64_t m = threadIdx.x; m < K; m += kBlock) {
        const int n = (int)(m / HWo);
        const int r = (int)(m - (int64_t)n * HWo);
        const int ho = r / g.Wo, wo = r - ho * g.Wo;
        const int h = ho * g.sH + kh * g.dH - g.pH;
        const int w = wo * g.sW + kw * g.dW - g.pW;
        if (h < 0 || h >= g.Hin || w < 0 || w >= g.Win) continue;
        a += (int32_t)qx[X.offset(n, ci, h, w)] * (int32_t)vq[G.offset(n, co, ho, wo)];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) a += __shfl_down(a, o);
    __shared__ int32_t part[kBlock / kWave];
    if (threadIdx.x % kWave == 0) part[threadIdx.x / kWave] = a;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kBlock / kWave; ++w) a += part[w];
        store_result(dW, e, dq2(a, *s_x, s_chan[co]), bf16);
        if (acc_out) acc_out[e] = a;
    }
}

}  // namespace

daq_status conv_fwd_generic(const daq_conv_desc& d, const int8_t* qx, const int8_t* qw, const float* s_x,
                            const float* s_w, float* Y, int32_t* acc, hipStream_t st) {
    daq_layout L;
    if (daq_layout_qx_nhwc(&d, &L) != DAQ_OK) return DAQ_ERR_INVALID_ARG;
    const Geo g = geo_of(d);
    const int64_t total = (int64_t)g.N * g.Cout * g.Ho * g.Wo;
    DAQ_LAUNCH("conv_fwd_direct", st,
               hipLaunchKernelGGL(k_fwd, dim3((unsigned)ceil_div(total, kBlock)), dim3(kBlock), 0, st, g,
                                  nhwc_view(L), qx, qw, s_x, s_w, Y, acc));
    return DAQ_OK;
}

daq_status conv_bwd_data_generic(const daq_conv_desc& d, const int8_t* qg, const float* s_g, const int8_t* qw,
                                 const float* s_w, float* dX, int32_t* acc, hipStream_t st, bool bf16) {
    daq_layout L;
    if (daq_layout_qg(&d, &L) != DAQ_OK) return DAQ_ERR_INVALID_ARG;
    const Geo g = geo_of(d);
    const int64_t total = (int64_t)g.N * g.Cin * g.Hin * g.Win;
    const dim3 grid((unsigned)ceil_div(total, kBlock));
    if (L.kind == DAQ_LAYOUT_NHWC)
        DAQ_LAUNCH("conv_bwd_data_direct", st,
                   hipLaunchKernelGGL((k_bwd_data<true>), grid, dim3(kBlock), 0, st, g, nhwc_view(L), CnhwView{}, qg,
                                      qw, s_g, s_w, dX, acc, bf16 ? 1 : 0));
    else
        DAQ_LAUNCH("conv_bwd_data_direct", st,
                   hipLaunchKernelGGL((k_bwd_data<false>), grid, dim3(kBlock), 0, st, g, NhwcView{}, cnhw_view(L), qg,
                                      qw, s_g, s_w, dX, acc, bf16 ? 1 : 0));
    return DAQ_OK;
}

daq_status conv_bwd_filter_generic(const daq_conv_desc& d, const int8_t* qx, const float* s_x, const int8_t* vq,
                                   const float* s_chan, float* dW, int32_t* acc, hipStream_t st, bool bf16) {
    daq_layout Lx, Lg;
    if (daq_layout_qx_cnhw(&d, &Lx) != DAQ_OK || daq_layout_vq(&d, &Lg) != DAQ_OK) return DAQ_ERR_INVALID_ARG;
    const Geo g = geo_of(d);
    const int64_t total = (int64_t)g.Cout * g.cig * g.kH * g.kW;
    DAQ_LAUNCH("conv_bwd_filter_direct", st,
               hipLaunchKernelGGL(k_bwd_filter, dim3((unsigned)total), dim3(kBlock), 0, st, g, cnhw_view(Lx),
                                  cnhw_view(Lg), qx, vq, s_x, s_chan, dW, acc, bf16 ? 1 : 0));
    return DAQ_OK;
}

}  // namespace daq
