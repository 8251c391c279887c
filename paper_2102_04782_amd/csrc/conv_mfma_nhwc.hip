// Channel-contracting int8 implicit GEMM on the gfx950 matrix cores: the data gradient
// q(G_X) = q(G) (.) q(W)  (Eq. "gx") and the forward convolution share it.
//
// The pixel operand is NHWC (the contraction axis, channels, is innermost), the filter operand is
// the packed [tap][row channel][contraction channel] copy.  The GEMM is computed transposed,
//
//     C[row channel][pixel] = sum over (tap, k)  Wp[tap][row][k] * P[src_pixel(pixel, tap)][k]
//
// so that an accumulator tile holds 16 consecutive pixels of one output channel per register and
// the fp32 NCHW result is written in 64-byte runs.  Each lane fetches the 16 contiguous channel
// bytes of its (pixel, tap) straight from global memory (L1/L2 absorb the tap re-reads) with
// out-of-image and stride-skipped taps predicated to zero; the filter chunk is staged in LDS and
// shared by the four waves.  A wave owns a 64 (rows) x 64 (pixels) tile, a workgroup 64 x 256.
#include "daq_internal.h"

namespace daq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kRows = 64;        // row channels per workgroup
constexpr int kPxWave = 64;      // pixels per wave
constexpr int kPxWg = 256;       // pixels per workgroup
constexpr int kKc = 64;          // contraction bytes per MFMA step
constexpr int kWPitch = kKc + 16;  // LDS pitch of a filter row: rotates banks between rows
constexpr int kTapGroup = 9;     // taps staged in LDS at a time

struct NhwcArgs {
    const int8_t* src;   // pixel operand, NHWC [N][Hs][Ws][cp]
    const int8_t* wpk;   // filter operand [taps][Crow][kp]
    int N, Hs, Ws, cp;   // source extents and channel pitch (the contraction length, multiple of 16)
    int Hd, Wd;          // extents of the result's spatial axes
    int Crow, kp;        // result channels; pitch of a filter row
    int kH, kW, sH, sW, pH, pW, dH, dW;
    int backward;        // 1: source pixel = (dst + pad - tap*dil) / stride when divisible; 0: dst*stride + tap*dil - pad
    int tiles_px;
    const float* s_a;
    const float* s_b;
    float* out;          // fp32 [N][Crow][Hd][Wd]
    int32_t* acc_out;    // optional raw accumulators, same shape
};

__global__ __launch_bounds__(256) void k_nhwc_mfma(NhwcArgs p) {
    __shared__ __align__(16) int8_t wl[kTapGroup * kRows * kWPitch];  // 46080 B

    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int li = lane & 15, lg = lane >> 4;
    const int tp = blockIdx.x % p.tiles_px;
    const int tr = blockIdx.x / p.tiles_px;
    const int row0 = tr * kRows;
    const int taps = p.kH * p.kW;
    const int HWd = p.Hd * p.Wd;
    const int64_t total_px = (int64_t)p.N * HWd;

    // the four 16-pixel groups of this lane's wave: image base, row, column
    int pn[4], ph[4], pw[4];
    bool pv[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int64_t P = (int64_t)tp * kPxWg + wave * kPxWave + b * 16 + li;
        pv[b] = P < total_px;
        const int64_t Pc = pv[b] ? P : 0;
        pn[b] = (int)(Pc / HWd);
        const int r = (int)(Pc - (int64_t)pn[b] * HWd);
        ph[b] = r / p.Wd;
        pw[b] = r - ph[b] * p.Wd;
    }

    v4i acc[4][4];
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[m][b] = v4i{0, 0, 0, 0};

    // 16 channel bytes of (pixel group b, tap, channel chunk kc) for this lane, or zeros
    auto load_b = [&](int tap, int kc, v4i (&out)[4]) {
        const int kh = tap / p.kW, kw = tap - kh * p.kW;
        const int k = kc + 16 * lg;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            int hs, ws;
            bool ok = pv[b] && k < p.cp;
            if (p.backward) {
                const int hn = ph[b] + p.pH - kh * p.dH, wn = pw[b] + p.pW - kw * p.dW;
                hs = hn / p.sH;
                ws = wn / p.sW;
                ok = ok && hn >= 0 && wn >= 0 && hs * p.sH == hn && ws * p.sW == wn && hs < p.Hs && ws < p.Ws;
            } else {
                hs = ph[b] * p.sH + kh * p.dH - p.pH;
                ws = pw[b] * p.sW + kw * p.dW - p.pW;
                ok = ok && hs >= 0 && ws >= 0 && hs < p.Hs && ws < p.Ws;
            }
            if (ok) {
                const int64_t off = (((int64_t)pn[b] * p.Hs + hs) * p.Ws + ws) * p.cp + k;
                out[b] = *reinterpret_cast<const v4i*>(p.src + off);
            } else {
                out[b] = v4i{0, 0, 0, 0};
            }
        }
    };

    const int nkc = (p.cp + kKc - 1) / kKc;
    v4i bcur[4], bnext[4];
    load_b(0, 0, bcur);

    for (int kci = 0; kci < nkc; ++kci) {
        const int kc = kci * kKc;
        for (int tg = 0; tg < taps; tg += kTapGroup) {
            const int tcount = min(kTapGroup, taps - tg);
            // stage Wp[tg .. tg+tcount)[row0 .. row0+64)[kc .. kc+64) into LDS
            __syncthreads();
            const int units = tcount * kRows * (kKc / 16);
            for (int u = tid; u < units; u += 256) {
                const int c16 = u & 3;
                const int row = (u >> 2) % kRows;
                const int t = (u >> 2) / kRows;
                const int rg = row0 + row, k = kc + 16 * c16;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (rg < p.Crow && k < p.kp)
                    v = *reinterpret_cast<const uint4*>(p.wpk + ((int64_t)(tg + t) * p.Crow + rg) * p.kp + k);
                *reinterpret_cast<uint4*>(wl + (t * kRows + row) * kWPitch + 16 * c16) = v;
            }
            __syncthreads();

            for (int t = 0; t < tcount; ++t) {
                // prefetch the pixel fragments of the next step while this one multiplies
                int ntap = tg + t + 1, nkc_i = kci;
                if (ntap == taps) { ntap = 0; ++nkc_i; }
                const bool more = nkc_i < nkc;
                if (more) load_b(ntap, nkc_i * kKc, bnext);

                v4i a[4];
#pragma unroll
                for (int m = 0; m < 4; ++m)
                    a[m] = *reinterpret_cast<const v4i*>(wl + (t * kRows + 16 * m + li) * kWPitch + 16 * lg);
#pragma unroll
                for (int m = 0; m < 4; ++m)
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        acc[m][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[m], bcur[b], acc[m][b], 0, 0, 0);
                if (more) {
#pragma unroll
                    for (int b = 0; b < 4; ++b) bcur[b] = bnext[b];
                }
            }
        }
    }

    // epilogue: register r of tile (m, b) is row 16m + 4*lg + r, pixel group b, pixel li
    const float scale = (*p.s_a / 127.0f) * (*p.s_b / 127.0f);
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        if (!pv[b]) continue;
#pragma unroll
        for (int m = 0; m < 4; ++m)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = row0 + 16 * m + 4 * lg + r;
                if (row < p.Crow) {
                    const int64_t off = (((int64_t)pn[b] * p.Crow + row) * p.Hd + ph[b]) * p.Wd + pw[b];
                    p.out[off] = (float)acc[m][b][r] * scale;
                    if (p.acc_out) p.acc_out[off] = acc[m][b][r];
                }
            }
    }
}

daq_status launch(NhwcArgs& a, hipStream_t st, const char* name) {
    const int64_t total_px = (int64_t)a.N * a.Hd * a.Wd;
    a.tiles_px = (int)ceil_div(total_px, kPxWg);
    const int tiles_r = (int)ceil_div(a.Crow, kRows);
    const dim3 grid((unsigned)((int64_t)a.tiles_px * tiles_r));
    DAQ_LAUNCH(name, st, hipLaunchKernelGGL(k_nhwc_mfma, grid, dim3(256), 0, st, a));
    return DAQ_OK;
}

}  // namespace

bool bwd_data_mfma_supported(const daq_conv_desc& d) { return d.groups == 1; }

daq_status conv_bwd_data_mfma(const daq_conv_desc& d, const int8_t* qg, const float* s_g, const int8_t* qw,
                              const float* s_w, float* dX, int32_t* acc, hipStream_t st) {
    daq_layout Lg;
    daq_wpack_layout Lw;
    if (daq_layout_qg(&d, &Lg) != DAQ_OK || daq_layout_qw(&d, &Lw) != DAQ_OK) return DAQ_ERR_INVALID_ARG;
    NhwcArgs a{};
    a.src = qg;
    a.wpk = qw + Lw.off_bwd;
    a.N = d.N; a.Hs = Lg.H; a.Ws = Lg.W; a.cp = Lg.c_pitch;
    a.Hd = d.Hin; a.Wd = d.Win;
    a.Crow = d.Cin; a.kp = Lw.cog_pitch;
    a.kH = d.kH; a.kW = d.kW; a.sH = d.strideH; a.sW = d.strideW; a.pH = d.padH; a.pW = d.padW;
    a.dH = d.dilH; a.dW = d.dilW;
    a.backward = 1;
    a.s_a = s_w; a.s_b = s_g;
    a.out = dX; a.acc_out = acc;
    return launch(a, st, "conv_bwd_data_mfma");
}

bool fwd_mfma_supported(const daq_conv_desc& d) { return d.groups == 1; }

daq_status conv_fwd_mfma(const daq_conv_desc& d, const int8_t* qx, const int8_t* qw, const float* s_x,
                         const float* s_w, float* Y, int32_t* acc, hipStream_t st) {
    daq_layout Lx;
    daq_wpack_layout Lw;
    if (daq_layout_qx_nhwc(&d, &Lx) != DAQ_OK || daq_layout_qw(&d, &Lw) != DAQ_OK) return DAQ_ERR_INVALID_ARG;
    NhwcArgs a{};
    a.src = qx;
    a.wpk = qw + Lw.off_fwd;
    a.N = d.N; a.Hs = d.Hin; a.Ws = d.Win; a.cp = Lx.c_pitch;
    a.Hd = daq_out_h(&d); a.Wd = daq_out_w(&d);
    a.Crow = d.Cout; a.kp = Lw.cig_pitch;
    a.kH = d.kH; a.kW = d.kW; a.sH = d.strideH; a.sW = d.strideW; a.pH = d.padH; a.pW = d.padW;
    a.dH = d.dilH; a.dW = d.dilW;
    a.backward = 0;
    a.s_a = s_x; a.s_b = s_w;
    a.out = Y; a.acc_out = acc;
    return launch(a, st, "conv_fwd_mfma");
}

}  // namespace daq
