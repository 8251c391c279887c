// 3-D convolution layers (the video-classification experiment: the depth axis is treated like height and width).
//
// Where the 3-D problem IS a 2-D problem - a filter that does not extend in height and width (time-only filters and
// pointwise layers: depth becomes the row axis and a whole frame the column axis), or a volume of depth one - the entry
// points hand it to the 2-D entry points, matrix-core kernels included; the views involved are pure reinterpretations of
// the NCDHW tensors.  Every other layer (3 x 3 x 3 and friends) runs on direct integer kernels: v_dot4_i32_i8 forms where
// the shapes allow it (k3_fwd_dot, k3_bwd_data_dot: 16 channels per load against filter rows that are uniform across the
// wave; k3_bwd_filter_dot: four positions of a row per load, unit stride and dilation along w, filters of at most
// 3 x 3 x 3), and one-multiply-at-a-time kernels for everything else.  The filter of such a layer is stored three times:
// plain [Cout][Cin/groups][taps], [tap][Cout][Cin/groups rounded up to 16] and [tap][Cin][Cout/groups rounded up to 16].
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

typedef int v4i3 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int32_t dot16(const v4i3& a, const v4i3& b, int32_t c) {
    c = __builtin_amdgcn_sdot4(a[0], b[0], c, false);
    c = __builtin_amdgcn_sdot4(a[1], b[1], c, false);
    c = __builtin_amdgcn_sdot4(a[2], b[2], c, false);
    return __builtin_amdgcn_sdot4(a[3], b[3], c, false);
}

constexpr int kCoT = 8;   // result channels per thread of the dot4 forms

// Layout of the three filter copies inside the q(W) buffer of a general 3-D layer.
struct W3 {
    int64_t off_fwd, off_bwd, bytes;
    int cigp, cogp;   // contraction lengths rounded up to 16
};
__host__ __device__ inline W3 w3_of(int Cout, int Cin, int groups, int taps) {
    W3 w{};
    const int cig = Cin / groups, cog = Cout / groups;
    w.cigp = (cig + 15) / 16 * 16;
    w.cogp = (cog + 15) / 16 * 16;
    const int64_t plain = ((int64_t)Cout * cig * taps + 255) / 256 * 256;
    w.off_fwd = plain;
    w.off_bwd = plain + ((int64_t)taps * Cout * w.cigp + 255) / 256 * 256;
    w.bytes = w.off_bwd + ((int64_t)taps * Cin * w.cogp + 255) / 256 * 256;
    return w;
}

// Forward, dot4 form: a thread owns one output position and kCoT consecutive result channels (blockIdx.y); per tap and 16
// input channels it loads 16 bytes of its pixel's NHWC record, and the kCoT filter rows it meets are the same for every
// lane of the wave (scalar loads).  Requires groups == 1, or whole 16-channel records and whole channel blocks per group.
__global__ __launch_bounds__(kBlock) void k3_fwd_dot(Geo3 g, NhwcView X, const int8_t* __restrict__ qx, const int8_t* __restrict__ wf,
                                                     int cigp, const float* s_x, const float* s_w, float* __restrict__ Y,
                                                     int32_t* __restrict__ acc_out) {
    const int64_t P = (int64_t)g.N * g.Do * g.Ho * g.Wo;
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const bool live = i < P;
    if (!live) i = 0;
    const int wo = (int)(i % g.Wo); i /= g.Wo;
    const int ho = (int)(i % g.Ho); i /= g.Ho;
    const int od = (int)(i % g.Do);
    const int n = (int)(i / g.Do);
    const int co0 = (int)blockIdx.y * kCoT;
    const int grp = co0 / g.cog;
    const int c16n = cigp / 16;
    int32_t a[kCoT];
#pragma unroll
    for (int j = 0; j < kCoT; ++j) a[j] = 0;
    for (int kd = 0; kd < g.kD; ++kd) {
        const int z = od * g.sD + kd * g.dD - g.pD;
        for (int kh = 0; kh < g.kH; ++kh) {
            const int h = ho * g.sH + kh * g.dH - g.pH;
            for (int kw = 0; kw < g.kW; ++kw) {
                const int w = wo * g.sW + kw * g.dW - g.pW;
                const bool ok = live && z >= 0 && z < g.Din && h >= 0 && h < g.Hin && w >= 0 && w < g.Win;
                const int8_t* xp = qx + (ok ? X.offset(n, grp * g.cig, z * g.Hin + h, w) : 0);
                const int tap = (kd * g.kH + kh) * g.kW + kw;
                for (int c = 0; c < c16n; ++c) {
                    v4i3 xv = *reinterpret_cast<const v4i3*>(xp + 16 * c);
                    if (!ok) xv = v4i3{0, 0, 0, 0};
#pragma unroll
                    for (int j = 0; j < kCoT; ++j) {
                        const int co = min(co0 + j, g.Cout - 1);   // uniform; rows past Cout are computed and dropped
                        const v4i3 wv = *reinterpret_cast<const v4i3*>(wf + ((int64_t)tap * g.Cout + co) * cigp + 16 * c);
                        a[j] = dot16(xv, wv, a[j]);
                    }
                }
            }
        }
    }
    if (!live) return;
    const int64_t vol = (int64_t)g.Do * g.Ho * g.Wo;
    const int64_t at0 = ((int64_t)n * g.Cout + co0) * vol + ((int64_t)od * g.Ho + ho) * g.Wo + wo;
#pragma unroll
    for (int j = 0; j < kCoT; ++j) {
        if (co0 + j >= g.Cout) break;
        Y[at0 + j * vol] = dq2(a[j], *s_x, *s_w);
        if (acc_out) acc_out[at0 + j * vol] = a[j];
    }
}

// Data gradient, dot4 form: a thread owns one input position and kCoT consecutive input channels; per tap whose output
// position exists it loads 16 gradient channels of that position's NHWC record.  Same requirements with the roles of
// the channel counts exchanged.
__global__ __launch_bounds__(kBlock) void k3_bwd_data_dot(Geo3 g, NhwcView G, const int8_t* __restrict__ qg, const int8_t* __restrict__ wb,
                                                          int cogp, const float* s_g, const float* s_w, float* __restrict__ dX,
                                                          int32_t* __restrict__ acc_out) {
    const int64_t P = (int64_t)g.N * g.Din * g.Hin * g.Win;
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const bool live = i < P;
    if (!live) i = 0;
    const int w = (int)(i % g.Win); i /= g.Win;
    const int h = (int)(i % g.Hin); i /= g.Hin;
    const int z = (int)(i % g.Din);
    const int n = (int)(i / g.Din);
    const int ci0 = (int)blockIdx.y * kCoT;
    const int grp = ci0 / g.cig;
    const int c16n = cogp / 16;
    int32_t a[kCoT];
#pragma unroll
    for (int j = 0; j < kCoT; ++j) a[j] = 0;
    for (int kd = 0; kd < g.kD; ++kd) {
        const int zn = z + g.pD - kd * g.dD;
        const bool zok = zn >= 0 && zn % g.sD == 0 && zn / g.sD < g.Do;
        for (int kh = 0; kh < g.kH; ++kh) {
            const int hn = h + g.pH - kh * g.dH;
            const bool hok = hn >= 0 && hn % g.sH == 0 && hn / g.sH < g.Ho;
            for (int kw = 0; kw < g.kW; ++kw) {
                const int wn = w + g.pW - kw * g.dW;
                const bool ok = live && zok && hok && wn >= 0 && wn % g.sW == 0 && wn / g.sW < g.Wo;
                const int8_t* gp = qg + (ok ? G.offset(n, grp * g.cog, (zn / g.sD) * g.Ho + hn / g.sH, wn / g.sW) : 0);
                const int tap = (kd * g.kH + kh) * g.kW + kw;
                for (int c = 0; c < c16n; ++c) {
                    v4i3 gv = *reinterpret_cast<const v4i3*>(gp + 16 * c);
                    if (!ok) gv = v4i3{0, 0, 0, 0};
#pragma unroll
                    for (int j = 0; j < kCoT; ++j) {
                        const int ci = min(ci0 + j, g.Cin - 1);   // uniform
                        const v4i3 wv = *reinterpret_cast<const v4i3*>(wb + ((int64_t)tap * g.Cin + ci) * cogp + 16 * c);
                        a[j] = dot16(gv, wv, a[j]);
                    }
                }
            }
        }
    }
    if (!live) return;
    const int64_t vol = (int64_t)g.Din * g.Hin * g.Win;
    const int64_t at0 = ((int64_t)n * g.Cin + ci0) * vol + ((int64_t)z * g.Hin + h) * g.Win + w;
#pragma unroll
    for (int j = 0; j < kCoT; ++j) {
        if (ci0 + j >= g.Cin) break;
        dX[at0 + j * vol] = dq2(a[j], *s_w, *s_g);
        if (acc_out) acc_out[at0 + j * vol] = a[j];
    }
}

// Four consecutive bytes from any address: the two aligned dwords around it, shifted (every plane ends in a zero halo, so
// the dword behind is addressable).
__device__ __forceinline__ uint32_t ld4_any(const int8_t* p) {
    const uintptr_t a = reinterpret_cast<uintptr_t>(p);
    const uint32_t* q = reinterpret_cast<const uint32_t*>(a & ~(uintptr_t)3);
    return __builtin_amdgcn_alignbyte(q[1], q[0], (uint32_t)(a & 3));
}

// Filter gradient, dot4 form: one workgroup per (co, input channel of its group) computes all taps of a filter of at most
// 3 x 3 x 3 at unit stride and dilation along w.  A thread takes rows (n, od, ho) of the gradient; per chunk of four
// positions it loads the gradient once and, per (kd, kh) whose activation row exists, the three shifted activation
// windows; positions whose tap falls into the padding are masked out of the gradient dword.
__global__ __launch_bounds__(kBlock) void k3_bwd_filter_dot(Geo3 g, CnhwView X, CnhwView G, const int8_t* __restrict__ qx,
                                                            const int8_t* __restrict__ vq, const float* s_x,
                                                            const float* __restrict__ s_chan, float* __restrict__ dW,
                                                            int32_t* __restrict__ acc_out) {
    __shared__ int32_t part[kBlock / kWave][27];
    const int cl = (int)blockIdx.x % g.cig, co = (int)blockIdx.x / g.cig;
    const int ci = (co / g.cog) * g.cig + cl;
    const int rows = g.N * g.Do * g.Ho;
    int32_t a[3][3][3];
#pragma unroll
    for (int kd = 0; kd < 3; ++kd)
#pragma unroll
        for (int kh = 0; kh < 3; ++kh)
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) a[kd][kh][kw] = 0;
    // byte masks of a chunk: position wo + i takes part in tap kw iff 0 <= wo + i + kw - pW < Win (and wo + i < Wo)
    for (int r = threadIdx.x; r < rows; r += kBlock) {
        const int ho = r % g.Ho, od = (r / g.Ho) % g.Do, n = r / (g.Ho * g.Do);
        const int8_t* grow = vq + G.offset(n, co, od * g.Ho + ho, 0);
        for (int wo = 0; wo < g.Wo; wo += 4) {
            const uint32_t g4 = ld4_any(grow + wo);
            uint32_t gm[3];
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                uint32_t m = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int w = wo + i + kw - g.pW;
                    if (wo + i < g.Wo && w >= 0 && w < g.Win) m |= 0xffu << (8 * i);
                }
                gm[kw] = g4 & m;
            }
#pragma unroll
            for (int kd = 0; kd < 3; ++kd) {
                const int z = od * g.sD + kd * g.dD - g.pD;
                if (kd >= g.kD || z < 0 || z >= g.Din) continue;
#pragma unroll
                for (int kh = 0; kh < 3; ++kh) {
                    const int h = ho * g.sH + kh * g.dH - g.pH;
                    if (kh >= g.kH || h < 0 || h >= g.Hin) continue;
                    // the windows of the three kw start one byte apart: all of them lie in three aligned dwords
                    const uintptr_t xa = reinterpret_cast<uintptr_t>(qx + X.offset(n, ci, z * g.Hin + h, 0) + wo - g.pW);
                    const uint32_t* q = reinterpret_cast<const uint32_t*>(xa & ~(uintptr_t)3);
                    const uint32_t q0 = q[0], q1 = q[1], q2 = q[2];
                    const uint32_t sh = (uint32_t)(xa & 3);
#pragma unroll
                    for (int kw = 0; kw < 3; ++kw) {
                        if (kw >= g.kW) continue;
                        const uint32_t sft = sh + kw;
                        const uint32_t x4 = __builtin_amdgcn_alignbyte(sft >= 4 ? q2 : q1, sft >= 4 ? q1 : q0, sft & 3);
                        a[kd][kh][kw] = __builtin_amdgcn_sdot4((int)gm[kw], (int)x4, a[kd][kh][kw], false);
                    }
                }
            }
        }
    }
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
#pragma unroll
    for (int kd = 0; kd < 3; ++kd)
#pragma unroll
        for (int kh = 0; kh < 3; ++kh)
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                int32_t v = a[kd][kh][kw];
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o);
                if (lane == 0) part[wave][(kd * 3 + kh) * 3 + kw] = v;
            }
    __syncthreads();
    const int t = threadIdx.x;
    if (t < 27) {
        const int kd = t / 9, kh = (t / 3) % 3, kw = t % 3;
        if (kd < g.kD && kh < g.kH && kw < g.kW) {
            int32_t v = 0;
            for (int w = 0; w < kBlock / kWave; ++w) v += part[w][t];
            const int64_t at = (((int64_t)co * g.cig + cl) * g.kD + kd) * g.kH * g.kW + kh * g.kW + kw;
            dW[at] = dq2(v, *s_x, s_chan[co]);
            if (acc_out) acc_out[at] = v;
        }
    }
}

// The two channel-contraction copies of the filter from its plain codes (the buffer behind the plain copy is zero).
__global__ __launch_bounds__(kBlock) void k3_pack_w(const int8_t* __restrict__ plain, int Cout, int Cin, int groups, int taps, W3 L,
                                                    int8_t* __restrict__ out) {
    const int cig = Cin / groups, cog = Cout / groups;
    const int64_t total = (int64_t)Cout * cig * taps;
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    const int tap = (int)(i % taps);
    const int cl = (int)((i / taps) % cig);
    const int co = (int)(i / ((int64_t)taps * cig));
    const int grp = co / cog;
    const int8_t code = plain[i];
    out[L.off_fwd + ((int64_t)tap * Cout + co) * L.cigp + cl] = code;
    out[L.off_bwd + ((int64_t)tap * Cin + grp * cig + cl) * L.cogp + co % cog] = code;
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

// Whether the dot4 forms serve a layer whose contraction runs over `kc` channels per group and whose result has `rc`
// channels per group: every 16-byte load must stay inside its group's channels (or there is a single group, whose
// record is zero padded), and a thread's block of result channels must not straddle two groups.
bool dot_channels_ok(int groups, int kc, int rc) { return groups == 1 || (kc % 16 == 0 && rc % kCoT == 0); }

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
    return w3_of(desc->Cout, desc->Cin, desc->groups, desc->kD * desc->kH * desc->kW).bytes;
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
    const Geo3 g = geo3_of(*desc);
    const int taps = g.kD * g.kH * g.kW;
    const W3 L3 = w3_of(g.Cout, g.Cin, g.groups, taps);
    const int64_t nw = elems_w(*desc), wb = L3.bytes;   // the plain codes, zeros behind them, then the two copies
    DAQ_LAUNCH("fill", st, hipLaunchKernelGGL(k3_zero, dim3(1), dim3(1), 0, st, bits));
    DAQ_LAUNCH("absmax", st, hipLaunchKernelGGL(k3_absmax, dim3((unsigned)std::min<int64_t>(ceil_div(nw, kBlock), 1024)), dim3(kBlock), 0, st, W, nw, bits));
    DAQ_LAUNCH("pack_w", st, hipLaunchKernelGGL(k3_quant_plain, dim3((unsigned)ceil_div(wb, kBlock)), dim3(kBlock), 0, st, W, nw, bits, s_w, qw, wb));
    DAQ_LAUNCH("pack_w", st, hipLaunchKernelGGL(k3_pack_w, dim3((unsigned)ceil_div(nw, kBlock)), dim3(kBlock), 0, st, qw, g.Cout, g.Cin,
                                                g.groups, taps, L3, qw));
    const int64_t px = (int64_t)g.N * g.Do * g.Ho * g.Wo;
    if (dot_channels_ok(g.groups, g.cig, g.cog) && ceil_div(px, kBlock) < ((int64_t)1 << 31) && ceil_div(g.Cout, kCoT) <= 65535) {
        const dim3 grid((unsigned)ceil_div(px, kBlock), (unsigned)ceil_div(g.Cout, kCoT));
        DAQ_LAUNCH("conv3d_fwd_dot", st,
                   hipLaunchKernelGGL(k3_fwd_dot, grid, dim3(kBlock), 0, st, g, nhwc_view(Ln), qx_nhwc, qw + L3.off_fwd, L3.cigp, s_x, s_w, Y,
                                      acc_out));
        return DAQ_OK;
    }
    const int64_t total = px * g.Cout;
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
    hipStream_t st = (hipStream_t)stream;
    const int64_t px = (int64_t)g.N * g.Din * g.Hin * g.Win;
    // the contraction runs over the output channels of a group here: the roles of the two channel counts are exchanged
    if (dot_channels_ok(g.groups, g.cog, g.cig) && ceil_div(px, kBlock) < ((int64_t)1 << 31) && ceil_div(g.Cin, kCoT) <= 65535) {
        const W3 L3 = w3_of(g.Cout, g.Cin, g.groups, g.kD * g.kH * g.kW);
        const dim3 grid((unsigned)ceil_div(px, kBlock), (unsigned)ceil_div(g.Cin, kCoT));
        DAQ_LAUNCH("conv3d_bwd_data_dot", st,
                   hipLaunchKernelGGL(k3_bwd_data_dot, grid, dim3(kBlock), 0, st, g, nhwc_view(Lg), qg, qw + L3.off_bwd, L3.cogp, s_global,
                                      s_w, dX, acc_out));
        return DAQ_OK;
    }
    const int64_t total = px * g.Cin;
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
    if (g.sW == 1 && g.dW == 1 && g.kD <= 3 && g.kH <= 3 && g.kW <= 3 && (int64_t)g.N * g.Do * g.Ho < ((int64_t)1 << 31) &&
        (int64_t)g.Cout * g.cig < ((int64_t)1 << 31)) {
        DAQ_LAUNCH("conv3d_bwd_filter_dot", st,
                   hipLaunchKernelGGL(k3_bwd_filter_dot, dim3((unsigned)(g.Cout * g.cig)), dim3(kBlock), 0, st, g, cnhw_view(Lx),
                                      cnhw_view(Lg), qx_cnhw, vq, s_x, s_chan, dW, acc_out));
        return DAQ_OK;
    }
    DAQ_LAUNCH("conv3d_bwd_filter_direct", st,
               hipLaunchKernelGGL(k3_bwd_filter, dim3((unsigned)elems_w(*desc)), dim3(kBlock), 0, st, g, cnhw_view(Lx), cnhw_view(Lg),
                                  qx_cnhw, vq, s_x, s_chan, dW, acc_out));
    return DAQ_OK;
}
