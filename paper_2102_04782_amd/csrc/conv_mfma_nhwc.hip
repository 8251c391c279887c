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
// out-of-image and stride-skipped taps predicated to zero, through a register ring nine steps deep
// so that the fetches of a whole 3x3 tap set are in flight together; the filter slices of those
// steps are staged in LDS and shared by the four waves.  A wave owns a 64 (rows) x 64 (pixels) tile,
// a workgroup 64 x 256.
#include "daq_internal.h"

namespace daq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kRows = 64;        // row channels per workgroup
constexpr int kPxWave = 64;      // pixels per wave
constexpr int kPxWg = 256;       // pixels per workgroup
constexpr int kKc = 64;          // contraction bytes per MFMA step
constexpr int kWPitch = kKc + 16;  // LDS pitch of a filter row: rotates banks between rows
constexpr int kRing = 9;         // (tap, channel chunk) steps in flight / staged at a time

// Exact unsigned division by an invariant divisor (Granlund-Montgomery round-up multiplier).
struct FastDiv {
    uint32_t mul;
    int32_t shift;
    int32_t one;
};
FastDiv make_fastdiv(uint32_t d) {
    FastDiv f{};
    f.one = (d == 1);
    int L = 0;
    while (((uint64_t)1 << L) < d) ++L;
    f.shift = L > 0 ? L - 1 : 0;
    f.mul = (uint32_t)((((uint64_t)1 << 32) * (((uint64_t)1 << L) - d)) / d + 1);
    return f;
}
__device__ __forceinline__ uint32_t fdiv(uint32_t x, const FastDiv& f) {
    if (f.one) return x;
    const uint32_t t = __umulhi(x, f.mul);
    return (t + ((x - t) >> 1)) >> f.shift;
}

constexpr int kMaxK = 8;  // largest filter extent the tap tables hold

struct NhwcArgs {
    const int8_t* src;   // pixel operand, NHWC [N][Hs][Ws][cp]
    const int8_t* wpk;   // filter operand [taps][Crow][kp]
    int N, Hs, Ws, cp;   // source extents and channel pitch (the contraction length, multiple of 16)
    int Hd, Wd;          // extents of the result's spatial axes
    int Crow, kp;        // result channels; pitch of a filter row
    int kH, kW, sH, sW, pH, pW, dH, dW;
    int backward;        // 1: source pixel = (dst + pad - tap*dil) / stride when divisible; 0: dst*stride + tap*dil - pad
    int tiles_px;
    // Source coordinate of (dst, tap) without a division in the kernel.  Per destination coordinate the
    // kernel keeps (A, R); per tap the host tabulates (dq, dr); source = A + dq, valid iff R == dr and
    // 0 <= source < extent.  forward: A = dst*stride - pad, R = 0, dq = tap*dil, dr = 0.
    // backward: A = (dst+pad)/stride, R = (dst+pad)%stride, dq = -(tap*dil/stride), dr = tap*dil%stride.
    int16_t dq_h[kMaxK], dr_h[kMaxK], dq_w[kMaxK], dr_w[kMaxK];
    FastDiv div_hw, div_w, div_sh, div_sw;
    const float* s_a;
    const float* s_b;
    float* out;          // fp32 [N][Crow][Hd][Wd]
    int32_t* acc_out;    // optional raw accumulators, same shape
};

// D = depth of the pixel-fragment register ring = number of (tap, channel chunk) steps whose filter
// slices are staged in LDS at a time.
template <int D>
__global__ __launch_bounds__(256, 2) void k_nhwc_mfma(NhwcArgs p) {
    __shared__ __align__(16) int8_t wl[D * kRows * kWPitch];

    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int li = lane & 15, lg = lane >> 4;
    const int tp = blockIdx.x % p.tiles_px;
    const int tr = blockIdx.x / p.tiles_px;
    const int row0 = tr * kRows;
    const int taps = p.kH * p.kW;
    const int HWd = p.Hd * p.Wd;
    const int64_t total_px = (int64_t)p.N * HWd;
    const int nkc = (p.cp + kKc - 1) / kKc;
    const int NS = nkc * taps;  // steps: channel chunk outer, tap inner

    // the four 16-pixel groups of this lane's wave: image base offset and the (A, R) pair of row and column
    int64_t pbase[4];
    int pn[4], ph[4], pw[4], ah[4], rh[4], aw[4], rw[4];
    bool pv[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int64_t P = (int64_t)tp * kPxWg + wave * kPxWave + b * 16 + li;
        pv[b] = P < total_px;
        const uint32_t Pc = pv[b] ? (uint32_t)P : 0u;
        pn[b] = (int)fdiv(Pc, p.div_hw);
        const uint32_t r = Pc - (uint32_t)pn[b] * (uint32_t)HWd;
        ph[b] = (int)fdiv(r, p.div_w);
        pw[b] = (int)r - ph[b] * p.Wd;
        pbase[b] = (int64_t)pn[b] * p.Hs * p.Ws * p.cp + 16 * lg;
        if (p.backward) {
            ah[b] = (int)fdiv((uint32_t)(ph[b] + p.pH), p.div_sh);
            rh[b] = ph[b] + p.pH - ah[b] * p.sH;
            aw[b] = (int)fdiv((uint32_t)(pw[b] + p.pW), p.div_sw);
            rw[b] = pw[b] + p.pW - aw[b] * p.sW;
        } else {
            ah[b] = ph[b] * p.sH - p.pH;
            rh[b] = 0;
            aw[b] = pw[b] * p.sW - p.pW;
            rw[b] = 0;
        }
    }

    v4i acc[4][4];
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[m][b] = v4i{0, 0, 0, 0};

    // 16 channel bytes of (pixel group b, tap (kh, kw), channel chunk kci) for this lane, or zeros
    auto load_b = [&](int kci, int kh, int kw, v4i (&out)[4]) {
        const int k = kci * kKc;
        const bool kok = k + 16 * lg < p.cp;
        const int dqh = p.dq_h[kh], drh = p.dr_h[kh], dqw = p.dq_w[kw], drw = p.dr_w[kw];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int hs = ah[b] + dqh, ws = aw[b] + dqw;
            const bool ok = pv[b] && kok && rh[b] == drh && rw[b] == drw && (unsigned)hs < (unsigned)p.Hs &&
                            (unsigned)ws < (unsigned)p.Ws;
            if (ok)
                out[b] = *reinterpret_cast<const v4i*>(p.src + pbase[b] + (int64_t)((hs * p.Ws + ws) * p.cp + k));
            else
                out[b] = v4i{0, 0, 0, 0};
        }
    };

    // Steps run channel chunk outer, (kh, kw) inner.  Two cursors walk them without divisions: one for
    // the step being fetched (D ahead), one for the filter slices being staged.
    int f_kci = 0, f_kh = 0, f_kw = 0, f_s = 0;
    auto fetch_advance = [&]() {
        ++f_s;
        if (++f_kw == p.kW) { f_kw = 0; if (++f_kh == p.kH) { f_kh = 0; ++f_kci; } }
    };
    // fill the ring: the pixel fragments of the first D steps are all in flight together
    v4i bf[D][4];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        if (f_s < NS) load_b(f_kci, f_kh, f_kw, bf[d]);
        fetch_advance();
    }

    const int srow = tid >> 2, sc16 = tid & 3;  // this thread stages 16 bytes of filter row srow for every step
    int w_kci = 0, w_tap = 0;
    for (int g0 = 0; g0 < NS; g0 += D) {
        __syncthreads();
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int rg = row0 + srow, k = w_kci * kKc + 16 * sc16;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (g0 + d < NS && rg < p.Crow && k < p.kp)
                v = *reinterpret_cast<const uint4*>(p.wpk + ((int64_t)w_tap * p.Crow + rg) * p.kp + k);
            *reinterpret_cast<uint4*>(wl + (d * kRows + srow) * kWPitch + 16 * sc16) = v;
            if (++w_tap == taps) { w_tap = 0; ++w_kci; }
        }
        __syncthreads();
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (g0 + d < NS) {
                v4i a[4];
#pragma unroll
                for (int m = 0; m < 4; ++m)
                    a[m] = *reinterpret_cast<const v4i*>(wl + (d * kRows + 16 * m + li) * kWPitch + 16 * lg);
#pragma unroll
                for (int m = 0; m < 4; ++m)
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        acc[m][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[m], bf[d][b], acc[m][b], 0, 0, 0);
                // this ring slot is free: fetch the fragments of the step D ahead
                if (f_s < NS) load_b(f_kci, f_kh, f_kw, bf[d]);
                fetch_advance();
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
    for (int k = 0; k < a.kH; ++k) {
        a.dq_h[k] = (int16_t)(a.backward ? -(k * a.dH / a.sH) : k * a.dH);
        a.dr_h[k] = (int16_t)(a.backward ? (k * a.dH) % a.sH : 0);
    }
    for (int k = 0; k < a.kW; ++k) {
        a.dq_w[k] = (int16_t)(a.backward ? -(k * a.dW / a.sW) : k * a.dW);
        a.dr_w[k] = (int16_t)(a.backward ? (k * a.dW) % a.sW : 0);
    }
    a.div_hw = make_fastdiv((uint32_t)(a.Hd * a.Wd));
    a.div_w = make_fastdiv((uint32_t)a.Wd);
    a.div_sh = make_fastdiv((uint32_t)a.sH);
    a.div_sw = make_fastdiv((uint32_t)a.sW);
    const int tiles_r = (int)ceil_div(a.Crow, kRows);
    const dim3 grid((unsigned)((int64_t)a.tiles_px * tiles_r));
    DAQ_LAUNCH(name, st, hipLaunchKernelGGL(k_nhwc_mfma<kRing>, grid, dim3(256), 0, st, a));
    return DAQ_OK;
}

}  // namespace

bool bwd_data_mfma_supported(const daq_conv_desc& d) { return d.groups == 1 && d.kH <= kMaxK && d.kW <= kMaxK; }

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

bool fwd_mfma_supported(const daq_conv_desc& d) { return d.groups == 1 && d.kH <= kMaxK && d.kW <= kMaxK; }

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
