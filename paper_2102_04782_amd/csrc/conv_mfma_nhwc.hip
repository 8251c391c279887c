// Channel-contracting int8 implicit GEMM on the gfx950 matrix cores: the data gradient
// q(G_X) = q(G) (.) q(W)  (Eq. "gx") and the forward convolution share it.  This is the per-tap
// re-staging form, which handles every stride; conv_mfma_halo.hip serves the layers its window
// scheme covers (unit stride, stride-2 data gradients) and is preferred there.
//
// The pixel operand is NHWC (the contraction axis, channels, is innermost), the filter operand is
// the packed [tap][row channel][contraction channel] copy.  The GEMM is computed transposed,
//
//     C[row channel][pixel] = sum over (tap, k)  Wp[tap][row][k] * P[src_pixel(pixel, tap)][k]
//
// so that an accumulator register holds 32 consecutive pixels of one output channel across 32 lanes
// and the fp32 NCHW result is written in 128-byte runs.
//
// One step = one (channel chunk of 64, tap).  Per step the workgroup stages a 256-pixel x 64-byte
// tile of the pixel operand (source pixels shifted by the tap; out-of-image and stride-skipped taps
// are zero) and a rows x 64-byte filter slice into LDS with coalesced 16-byte loads (four adjacent
// lanes fetch one pixel's 64 bytes), double buffered, through a register ring that keeps the
// fetches of the next kRing steps in flight.  The waves multiply with v_mfma_i32_32x32x32_i8
// (measured at twice the rate of the 16x16x64 form on this chip); fragments are read from LDS as
// aligned 16-byte vectors, rows padded to 80 bytes so that eight lanes cover all banks.
//
// All per-tap index work is hoisted: a thread keeps, for each of the four pixels it stages, a base
// offset and a bit mask of the taps that hit the image; a tap then only adds a uniform offset.
#include "daq_internal.h"

namespace daq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kPxWg = 256;         // pixels per workgroup
constexpr int kKc = 64;            // contraction bytes per step (two MFMA K-steps of 32)
constexpr int kPitch = kKc + 16;   // LDS pitch of a staged row
constexpr int kRing = 4;           // steps whose global loads are in flight beyond the one being staged
constexpr int kMaxK = 8;           // largest filter extent (tap masks hold 64 taps)

struct NhwcArgs {
    const int8_t* src;   // pixel operand, NHWC [N][Hs][Ws][cp]
    const int8_t* wpk;   // filter operand [taps][Crow][kp]
    uint32_t src_bytes, wpk_bytes;  // extents of the two buffers (below 2^31: offsets are 32-bit)
    int N, Hs, Ws, cp;   // source extents and channel pitch (the contraction length, multiple of 16)
    int Hd, Wd;          // extents of the result's spatial axes
    int Crow, kp;        // result channels; pitch of a filter row
    int kH, kW, sH, sW, pH, pW;
    int backward;        // 1: data gradient (source = (dst + pad - tap*dil) / stride when divisible); 0: forward
    int tiles_px;
    // Source coordinate of (dst, tap) without a division in the kernel.  Per destination coordinate the
    // kernel keeps (A, R); per tap the host tabulates (dq, dr); source = A + dq, valid iff R == dr and
    // 0 <= source < extent.  forward: A = dst*stride - pad, R = 0, dq = tap*dil, dr = 0.
    // backward: A = (dst+pad)/stride, R = (dst+pad)%stride, dq = -(tap*dil/stride), dr = tap*dil%stride.
    // 32-bit entries: a uniform index then costs a scalar load, not a vector-memory round trip.
    int dq_h[kMaxK], dr_h[kMaxK], dq_w[kMaxK], dr_w[kMaxK];
    int tap_off[kMaxK * kMaxK];  // (dq_h*Ws + dq_w)*cp: byte offset a tap adds to a pixel's anchor
    FastDiv div_hw, div_w, div_sh, div_sw;
    const float* s_a;
    const float* s_b;
    float* out;          // fp32 [N][Crow][Hd][Wd]
    int32_t* acc_out;    // optional raw accumulators, same shape
    int bf16;            // the result is bfloat16 storage
};

constexpr uint32_t kOob = 0x80000000u;  // a buffer offset past every extent: such a load returns zeros

__device__ __forceinline__ v4i buffer_load16(__amdgpu_buffer_rsrc_t rsrc, uint32_t voffset, uint32_t soffset) {
    return __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voffset, (int)soffset, 0);
}

// WR = waves along the row (output channel) axis: 1 -> 64 rows x 256 pixels per workgroup with
// 64 x 64 wave tiles, 2 -> 128 rows x 256 pixels with 64 x 128 wave tiles.
template <int WR>
__global__ __launch_bounds__(256) void k_nhwc_mfma(NhwcArgs p) {
    constexpr int ROWS = 64 * WR;
    constexpr int WPX = 4 / WR;               // waves along pixels
    constexpr int PXW = kPxWg / WPX;          // pixels per wave
    constexpr int BF = PXW / 32;              // pixel fragments per wave
    constexpr int A_PER_T = ROWS * 4 / 256;   // 16-byte units of the filter slice per thread
    constexpr int A_BYTES = ROWS * kPitch;
    constexpr int STAGE = A_BYTES + kPxWg * kPitch;
    __shared__ __align__(16) int8_t lds[2 * STAGE];

    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int l32 = lane & 31, lh = lane >> 5;
    const int wr = wave % WR, wp = wave / WR;
    const int tp = blockIdx.x % p.tiles_px;
    const int tr = blockIdx.x / p.tiles_px;
    const int row0 = tr * ROWS;
    const int taps = p.kH * p.kW;
    const int HWd = p.Hd * p.Wd;
    const uint32_t total_px = (uint32_t)p.N * (uint32_t)HWd;
    const int nkc = (p.cp + kKc - 1) / kKc;
    const int NS = nkc * taps;  // steps: channel chunk outer, tap inner

    // Both operands are read through buffer descriptors: an offset of kOob returns zeros, which is how
    // padding taps, stride-skipped taps and ragged tiles are handled without branches or selects.
    const __amdgpu_buffer_rsrc_t rs_src = __builtin_amdgcn_make_buffer_rsrc((void*)p.src, 0, (int)p.src_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc((void*)p.wpk, 0, (int)p.wpk_bytes, 0x00020000);

    // ---- staging assignment: this thread fetches chunk sc (16 bytes) of pixels spx + 64*i ----
    const int sc = tid & 3, spx = tid >> 2;
    uint32_t poff[4];        // byte offset of the pixel's source anchor (A_h, A_w), plus the chunk
    uint32_t pm_lo[4], pm_hi[4];  // bit t set: tap t reads inside the image for this pixel
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t P = (uint32_t)tp * kPxWg + spx + 64 * i;
        const bool pv = P < total_px;
        const uint32_t Pc = pv ? P : 0u;
        const int n = (int)fdiv(Pc, p.div_hw);
        const uint32_t r = Pc - (uint32_t)n * (uint32_t)HWd;
        const int h = (int)fdiv(r, p.div_w);
        const int w = (int)r - h * p.Wd;
        int ah, rh, aw, rw;
        if (p.backward) {
            ah = (int)fdiv((uint32_t)(h + p.pH), p.div_sh);
            rh = h + p.pH - ah * p.sH;
            aw = (int)fdiv((uint32_t)(w + p.pW), p.div_sw);
            rw = w + p.pW - aw * p.sW;
        } else {
            ah = h * p.sH - p.pH;
            rh = 0;
            aw = w * p.sW - p.pW;
            rw = 0;
        }
        poff[i] = (uint32_t)(((n * p.Hs + ah) * p.Ws + aw) * p.cp + 16 * sc);
        // separable validity: rows that hit the image, columns that hit the image
        uint32_t hm = 0, wm = 0;
#pragma unroll
        for (int k = 0; k < kMaxK; ++k) {
            const bool hok = k < p.kH && rh == p.dr_h[k] && (unsigned)(ah + p.dq_h[k]) < (unsigned)p.Hs;
            const bool wok = k < p.kW && rw == p.dr_w[k] && (unsigned)(aw + p.dq_w[k]) < (unsigned)p.Ws;
            hm |= (uint32_t)hok << k;
            wm |= (uint32_t)wok << k;
        }
        uint64_t m = 0;
#pragma unroll
        for (int k = 0; k < kMaxK; ++k)
            if (k < p.kH) m |= ((hm >> k) & 1u) ? ((uint64_t)wm << (k * p.kW)) : 0ull;
        if (!pv) m = 0;
        pm_lo[i] = (uint32_t)m;
        pm_hi[i] = (uint32_t)(m >> 32);
    }
    // filter slice: unit j of this thread is row srow + 64*j, chunk sc
    const int srow = tid >> 2;
    uint32_t woff[A_PER_T];
#pragma unroll
    for (int j = 0; j < A_PER_T; ++j) {
        const int rg = row0 + srow + 64 * j;
        woff[j] = rg < p.Crow ? (uint32_t)(rg * p.kp + 16 * sc) : kOob;
    }

    // cursor over the steps being fetched (uniform)
    int f_tap = 0, f_k = 0, f_s = 0;
    v4i ra[kRing][A_PER_T], rb[kRing][4];
    // Always issues the same number of loads (past the last step they are out of bounds and return
    // zeros), so the compiler can count outstanding loads exactly and the ring stays kRing steps deep.
    auto fetch = [&](int slot) {
        const bool live = f_s < NS;
        const int tap = live ? f_tap : 0;
        const uint32_t toff = (uint32_t)p.tap_off[tap];
        const uint32_t bit_lo = tap < 32 ? (1u << tap) : 0u, bit_hi = tap >= 32 ? (1u << (tap - 32)) : 0u;
        const bool kok_b = live && f_k + 16 * sc < p.cp;
        const bool kok_a = live && f_k + 16 * sc < p.kp;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bool ok = kok_b && (((pm_lo[i] & bit_lo) | (pm_hi[i] & bit_hi)) != 0u);
            rb[slot][i] = buffer_load16(rs_src, ok ? poff[i] + toff : kOob, (uint32_t)f_k);
        }
        const uint32_t wbase = (uint32_t)(tap * p.Crow * p.kp + f_k);
#pragma unroll
        for (int j = 0; j < A_PER_T; ++j) ra[slot][j] = buffer_load16(rs_w, kok_a ? woff[j] : kOob, wbase);
        ++f_s;
        if (++f_tap == taps) { f_tap = 0; f_k += kKc; }
    };
    auto stage = [&](int buf, int slot) {
        int8_t* A = lds + buf * STAGE;
        int8_t* B = A + A_BYTES;
#pragma unroll
        for (int j = 0; j < A_PER_T; ++j)
            *reinterpret_cast<v4i*>(A + (srow + 64 * j) * kPitch + 16 * sc) = ra[slot][j];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *reinterpret_cast<v4i*>(B + (spx + 64 * i) * kPitch + 16 * sc) = rb[slot][i];
    };

    v16i acc[2][BF];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < BF; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0;

    // prologue: step 0 into LDS, steps 1..kRing in flight
    fetch(0);
    stage(0, 0);
#pragma unroll
    for (int d = 1; d <= kRing; ++d) fetch(d % kRing);
    __syncthreads();

    for (int base = 0; base < NS; base += kRing) {
#pragma unroll
        for (int u = 0; u < kRing; ++u) {
            const int s = base + u;
            if (s < NS) {  // uniform; only the multiplies are skipped on the padded tail steps
                const int8_t* A = lds + (s & 1) * STAGE + (wr * 64 + l32) * kPitch + 16 * lh;
                const int8_t* B = lds + (s & 1) * STAGE + A_BYTES + (wp * PXW + l32) * kPitch + 16 * lh;
#pragma unroll
                for (int sub = 0; sub < 2; ++sub) {
                    v4i a[2], b[BF];
#pragma unroll
                    for (int x = 0; x < 2; ++x) a[x] = *reinterpret_cast<const v4i*>(A + x * 32 * kPitch + 32 * sub);
#pragma unroll
                    for (int y = 0; y < BF; ++y) b[y] = *reinterpret_cast<const v4i*>(B + y * 32 * kPitch + 32 * sub);
#pragma unroll
                    for (int x = 0; x < 2; ++x)
#pragma unroll
                        for (int y = 0; y < BF; ++y)
                            acc[x][y] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[x], b[y], acc[x][y], 0, 0, 0);
                }
            }
            // step s+1 moves from its ring slot to the other LDS buffer; the slot is refilled kRing steps ahead
            const int nslot = (u + 1) % kRing;
            stage((s + 1) & 1, nslot);
            fetch(nslot);
            __syncthreads();
        }
    }

    // epilogue: register r of tile (x, y) is row 32x + 8*(r/4) + 4*lh + r%4, pixel 32y + l32
    const float scale = (*p.s_a / 127.0f) * (*p.s_b / 127.0f);
    const int rowbase = row0 + wr * 64 + 4 * lh;
    const bool full_rows = row0 + ROWS <= p.Crow;
#pragma unroll
    for (int y = 0; y < BF; ++y) {
        const uint32_t P = (uint32_t)tp * kPxWg + wp * PXW + 32 * y + l32;
        if (P >= total_px) continue;
        const int n = (int)fdiv(P, p.div_hw);
        const uint32_t rem = P - (uint32_t)n * (uint32_t)HWd;
        const int64_t pix = ((int64_t)n * p.Crow + rowbase) * HWd + rem;
        float* o = p.out + pix;
        if (p.bf16) {   // uniform: the narrow result, one 2-byte store per value
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int dr = 32 * x + 8 * (r >> 2) + (r & 3);
                    if (rowbase + dr < p.Crow) store_result(p.out, pix + (int64_t)dr * HWd, (float)acc[x][y][r] * scale, 1);
                }
        } else if (full_rows) {
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[(32 * x + 8 * (r >> 2) + (r & 3)) * HWd] = (float)acc[x][y][r] * scale;
        } else {
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int dr = 32 * x + 8 * (r >> 2) + (r & 3);
                    if (rowbase + dr < p.Crow) o[dr * HWd] = (float)acc[x][y][r] * scale;
                }
        }
        if (p.acc_out) {
            int32_t* ao = p.acc_out + pix;
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int dr = 32 * x + 8 * (r >> 2) + (r & 3);
                    if (rowbase + dr < p.Crow) ao[dr * HWd] = acc[x][y][r];
                }
        }
    }
}

daq_status launch(NhwcArgs& a, int dH, int dW, hipStream_t st, const char* name) {
    const int64_t total_px = (int64_t)a.N * a.Hd * a.Wd;
    a.tiles_px = (int)ceil_div(total_px, kPxWg);
    for (int k = 0; k < kMaxK; ++k) a.dq_h[k] = a.dr_h[k] = a.dq_w[k] = a.dr_w[k] = 0;
    for (int k = 0; k < a.kH; ++k) {
        a.dq_h[k] = a.backward ? -(k * dH / a.sH) : k * dH;
        a.dr_h[k] = a.backward ? (k * dH) % a.sH : 0;
    }
    for (int k = 0; k < a.kW; ++k) {
        a.dq_w[k] = a.backward ? -(k * dW / a.sW) : k * dW;
        a.dr_w[k] = a.backward ? (k * dW) % a.sW : 0;
    }
    for (int t = 0; t < a.kH * a.kW; ++t) a.tap_off[t] = (a.dq_h[t / a.kW] * a.Ws + a.dq_w[t % a.kW]) * a.cp;
    a.div_hw = make_fastdiv((uint32_t)(a.Hd * a.Wd));
    a.div_w = make_fastdiv((uint32_t)a.Wd);
    a.div_sh = make_fastdiv((uint32_t)a.sH);
    a.div_sw = make_fastdiv((uint32_t)a.sW);
    if (a.Crow > 64) {
        const dim3 grid((unsigned)((int64_t)a.tiles_px * ceil_div(a.Crow, 128)));
        DAQ_LAUNCH(name, st, hipLaunchKernelGGL(k_nhwc_mfma<2>, grid, dim3(256), 0, st, a));
    } else {
        const dim3 grid((unsigned)a.tiles_px);
        DAQ_LAUNCH(name, st, hipLaunchKernelGGL(k_nhwc_mfma<1>, grid, dim3(256), 0, st, a));
    }
    return DAQ_OK;
}

bool nhwc_supported(const daq_conv_desc& d) {
    if (d.groups != 1 || d.kH > kMaxK || d.kW > kMaxK) return false;
    daq_layout Lx, Lg;
    daq_wpack_layout Lw;
    if (daq_layout_qx_nhwc(&d, &Lx) != DAQ_OK || daq_layout_qg(&d, &Lg) != DAQ_OK || daq_layout_qw(&d, &Lw) != DAQ_OK)
        return false;
    const int64_t lim = (int64_t)1 << 31;  // 32-bit buffer offsets
    return Lx.bytes < lim && Lg.bytes < lim && Lw.bytes < lim;
}

}  // namespace

bool bwd_data_mfma_supported(const daq_conv_desc& d) { return nhwc_supported(d); }

daq_status conv_bwd_data_mfma(const daq_conv_desc& d, const int8_t* qg, const float* s_g, const int8_t* qw,
                              const float* s_w, float* dX, int32_t* acc, hipStream_t st, bool bf16) {
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
    a.backward = 1;
    a.s_a = s_w; a.s_b = s_g;
    a.out = dX; a.acc_out = acc;
    a.bf16 = bf16 ? 1 : 0;
    a.src_bytes = (uint32_t)Lg.bytes;
    a.wpk_bytes = (uint32_t)(Lw.bytes - Lw.off_bwd);
    return launch(a, d.dilH, d.dilW, st, "conv_bwd_data_nhwc");
}

bool fwd_mfma_supported(const daq_conv_desc& d) { return nhwc_supported(d); }

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
    a.backward = 0;
    a.s_a = s_x; a.s_b = s_w;
    a.out = Y; a.acc_out = acc;
    a.src_bytes = (uint32_t)Lx.bytes;
    a.wpk_bytes = (uint32_t)(Lw.bytes - Lw.off_fwd);
    return launch(a, d.dilH, d.dilW, st, "conv_fwd_nhwc");
}

}  // namespace daq
