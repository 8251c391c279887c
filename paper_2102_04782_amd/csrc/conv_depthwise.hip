// Depthwise (groups = channels) backward convolutions on channel-major int8 planes.
//
// With one input and one output channel per group there is no contraction over channels, so the
// matrix cores have nothing to do: both products are bandwidth bound (data gradient: 1 byte read and
// 4 written per element; filter gradient: 2 bytes read per element) and run on v_dot4_i32_i8.
//
// Both kernels lean on the plane layout: images sit in pitched slots whose spare rows / columns are
// zero and every plane starts and ends with a zero halo, so a neighbour a filter tap reaches outside
// the image is an addressable zero and no bounds test is needed anywhere.
#include <algorithm>

#include "daq_internal.h"

namespace daq {

namespace {

constexpr int kBlock = 256;
constexpr int kMaxK = 7;            // largest filter extent of the general data-gradient kernel
constexpr int kDwSlabBytes = 4096;  // bytes of the flat axis one filter-gradient workgroup covers per iteration

typedef int v2i_a4 __attribute__((ext_vector_type(2), aligned(4)));
typedef int v4i_a4 __attribute__((ext_vector_type(4), aligned(4)));
typedef int v4i __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int dot4(int a, int b, int c) { return __builtin_amdgcn_sdot4(a, b, c, false); }

// The 8 bytes at base + off (any byte alignment, off may be negative inside the zero halo).  A byte-aligned vector
// load runs at half the rate of a dword-aligned one on this chip, so 12 bytes are fetched from the dword below and
// shifted; base must be dword aligned.
__device__ __forceinline__ void load8(const int8_t* base, int64_t off, unsigned& lo, unsigned& hi) {
    const int8_t* src = base + (off & ~(int64_t)3);
    const unsigned sh = (unsigned)(off & 3);
    const v2i_a4 d01 = *reinterpret_cast<const v2i_a4*>(src);
    const unsigned d2 = *reinterpret_cast<const unsigned*>(src + 8);
    lo = __builtin_amdgcn_alignbyte((unsigned)d01[1], (unsigned)d01[0], sh);
    hi = __builtin_amdgcn_alignbyte(d2, (unsigned)d01[1], sh);
}

typedef float v4f __attribute__((ext_vector_type(4)));

struct DxArgs {
    const int8_t* qg;      // planar gradient, [C][chan_pitch]
    const int8_t* qw;      // plain filter copy, [C][kH*kW]
    int64_t chan_pitch;
    int lead, img_rows, row_pitch;
    int N, C, Hin, Win;
    int kH, kW, pH, pW, dH, dW;
    int s_log2;            // log2 of the (square, power-of-two) stride
    FastDiv div_wq, div_h, div_c;
    int wq;                // quads of output columns per row
    FastDiv div_hq;        // block kernel: by hq
    int hq;                // block kernel: quads of output rows per plane
    int Ho;                // block kernel: rows of the gradient
    const float* s_g;      // one scale, or one per channel (per_chan)
    const float* s_w;
    int per_chan;          // the gradient is the per-channel copy: channel c is de-quantized with s_g[c]
    int flip;              // 3 x 3 kernels at unit stride: apply the filter rotated by 180 degrees - the forward convolution of a
                           // 3 x 3, padding-1 layer is its data gradient with the rotated filter (planes are then activations)
    float* dX;
    int32_t* acc_out;
    int nt;                // large result: streaming stores
    int bf16;              // dX is bfloat16 storage
};

// Data gradient, unit stride and dilation, kW <= 4: a thread produces four adjacent outputs of one row.
// For filter row kh it reads the 8 gradient bytes that cover the windows of all four outputs with one
// (byte-aligned) load, and each output is one dot4 of its 4-byte window with the reversed filter row.
// KH = KW = 3 is instantiated with constant extents (every load issued up front, filter rows fetched as dwords);
// KH = 0 takes the extents from the arguments.
template <int KH, int KW>
__global__ __launch_bounds__(kBlock) void k_dwise_dx_unit(DxArgs p) {
    const int kH = KH ? KH : p.kH, kW = KW ? KW : p.kW;
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    const uint32_t rows = (uint32_t)p.N * p.C * p.Hin;
    const uint32_t row = fdiv(i, p.div_wq);
    if (row >= rows) return;
    const int w0 = 4 * (int)(i - row * (uint32_t)p.wq);
    const uint32_t nc = fdiv(row, p.div_h);
    const int h = (int)(row - nc * (uint32_t)p.Hin);
    const uint32_t n = fdiv(nc, p.div_c);
    const int c = (int)(nc - n * (uint32_t)p.C);

    const int8_t* g = p.qg + (int64_t)c * p.chan_pitch + p.lead;
    const int8_t* wrow = p.qw + c * (kH * kW);
    int acc[4] = {0, 0, 0, 0};
#pragma unroll
    for (int kh = 0; kh < kH; ++kh) {
        // reversed filter row in one dword: byte m = W[kh][kW-1-m], zero beyond kW
        int wr = 0;
        if (KW == 3) {
            // bytes W0 W1 W2 and one byte of whatever follows (the packed filter has further copies behind this one)
            typedef int i1 __attribute__((ext_vector_type(1), aligned(1)));
            const int raw = (*reinterpret_cast<const i1*>(wrow + (p.flip ? 2 - kh : kh) * 3))[0];
            wr = (int)__builtin_amdgcn_perm(0u, (unsigned)raw, p.flip ? 0x0c020100u : 0x0c000102u);   // flip: see DxArgs
        } else {
            for (int m = 0; m < kW; ++m) wr |= ((int)(uint8_t)wrow[kh * kW + (kW - 1 - m)]) << (8 * m);
        }
        const int ho = h + p.pH - kh;
        const int col0 = w0 + p.pW - (kW - 1);
        unsigned lo, hi;
        load8(g, (int64_t)((int)n * p.img_rows + ho) * p.row_pitch + col0, lo, hi);
        acc[0] = dot4((int)lo, wr, acc[0]);
        acc[1] = dot4((int)__builtin_amdgcn_alignbyte(hi, lo, 1), wr, acc[1]);
        acc[2] = dot4((int)__builtin_amdgcn_alignbyte(hi, lo, 2), wr, acc[2]);
        acc[3] = dot4((int)__builtin_amdgcn_alignbyte(hi, lo, 3), wr, acc[3]);
    }
    const float scale = (*p.s_w / 127.0f) * (p.s_g[p.per_chan ? c : 0] / 127.0f);
    const int64_t o = (int64_t)row * p.Win + w0;
    if (w0 + 4 <= p.Win && ((p.Win & 3) == 0)) {
        store_result4(p.dX, o, (float)acc[0] * scale, (float)acc[1] * scale, (float)acc[2] * scale, (float)acc[3] * scale, p.bf16, p.nt);
        if (p.acc_out) *reinterpret_cast<int4*>(p.acc_out + o) = make_int4(acc[0], acc[1], acc[2], acc[3]);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (w0 + j < p.Win) {
                store_result(p.dX, o + j, (float)acc[j] * scale, p.bf16);
                if (p.acc_out) p.acc_out[o + j] = acc[j];
            }
    }
}

// Data gradient, stride 2 or 4, unit dilation: a thread produces four adjacent outputs w0..w0+3 (w0 a multiple
// of four).  For a live filter row (h + pad - kh a multiple of the stride) the gradient columns the four outputs
// can touch lie within 8 bytes, fetched with one load.  Which taps are live for output j, and which of the 8
// bytes they read, depends only on (j + pad - kw) - the same for every thread - so the selection is scalar
// control flow and the work per live tap is one byte extract and one multiply-add.
// SLOG2 / PAD >= 0 fix log2(stride) and the padding at compile time: the tap selection below then folds to constants
// (the 3 x 3, stride 2, pad 1 layers of MobileNetV2 spend their time here).
template <int KH, int KW, int SLOG2, int PAD>
__global__ __launch_bounds__(kBlock) void k_dwise_dx_strided(DxArgs p) {
    const int kH = KH ? KH : p.kH, kW = KW ? KW : p.kW;
    const int s_log2 = SLOG2 >= 0 ? SLOG2 : p.s_log2;
    const int pH = PAD >= 0 ? PAD : p.pH, pW = PAD >= 0 ? PAD : p.pW;
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    const uint32_t rows = (uint32_t)p.N * p.C * p.Hin;
    const uint32_t row = fdiv(i, p.div_wq);
    if (row >= rows) return;
    const int w0 = 4 * (int)(i - row * (uint32_t)p.wq);
    const uint32_t nc = fdiv(row, p.div_h);
    const int h = (int)(row - nc * (uint32_t)p.Hin);
    const uint32_t n = fdiv(nc, p.div_c);
    const int c = (int)(nc - n * (uint32_t)p.C);

    const int8_t* g = p.qg + (int64_t)c * p.chan_pitch + p.lead;
    const int8_t* wf = p.qw + c * (kH * kW);
    const int smask = (1 << s_log2) - 1;
    // first gradient column any of the four outputs can read, relative to w0 >> s_log2 (an arithmetic shift: floor)
    const int c_first = (pW - (kW - 1)) >> s_log2;
    int acc[4] = {0, 0, 0, 0};
#pragma unroll
    for (int kh = 0; kh < kH; ++kh) {
        const int th = h + pH - kh;
        if (th & smask) continue;
        unsigned v[2];
        load8(g, (int64_t)((int)n * p.img_rows + (th >> s_log2)) * p.row_pitch + (w0 >> s_log2) + c_first, v[0], v[1]);
#pragma unroll
        for (int kw = 0; kw < kW; ++kw) {
            const int wv = wf[kh * kW + kw];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int t = j + pW - kw;              // uniform
                if (t & smask) continue;
                const int b = (t >> s_log2) - c_first;   // uniform byte index, 0..7
                const int word = (int)(b < 4 ? v[0] : v[1]);
                acc[j] += __builtin_amdgcn_sbfe(word, 8 * (b & 3), 8) * wv;
            }
        }
    }
    const float scale = (*p.s_w / 127.0f) * (p.s_g[p.per_chan ? c : 0] / 127.0f);
    const int64_t o = (int64_t)row * p.Win + w0;
    if (w0 + 4 <= p.Win && ((p.Win & 3) == 0)) {
        store_result4(p.dX, o, (float)acc[0] * scale, (float)acc[1] * scale, (float)acc[2] * scale, (float)acc[3] * scale, p.bf16, p.nt);
        if (p.acc_out) *reinterpret_cast<int4*>(p.acc_out + o) = make_int4(acc[0], acc[1], acc[2], acc[3]);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (w0 + j < p.Win) {
                store_result(p.dX, o + j, (float)acc[j] * scale, p.bf16);
                if (p.acc_out) p.acc_out[o + j] = acc[j];
            }
    }
}

// Data gradient, 3 x 3, unit stride and dilation, padding 1, row length a multiple of four: a thread produces a 4 x 4
// block of outputs from the six gradient rows h0-1 .. h0+4 it touches.  Each row is fetched once (8 bytes from column
// w0-1), its four 4-byte windows are derived once, and it feeds the up to three output rows that read it: the same
// dot4 per (output, filter row) as the row kernel above with half the loads and shifts and a quarter of the index
// arithmetic per output.  Rows past the image are never needed for a stored output; their index is clamped to the
// zero row that follows every image.
__global__ __launch_bounds__(kBlock) void k_dwise_dx_unit_block(DxArgs p) {
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    const uint32_t rq = fdiv(i, p.div_wq);
    const int w0 = 4 * (int)(i - rq * (uint32_t)p.wq);
    const uint32_t nc = fdiv(rq, p.div_hq);
    if (nc >= (uint32_t)p.N * p.C) return;
    const int h0 = 4 * (int)(rq - nc * (uint32_t)p.hq);
    const uint32_t n = fdiv(nc, p.div_c);
    const int c = (int)(nc - n * (uint32_t)p.C);

    const int8_t* g = p.qg + (int64_t)c * p.chan_pitch + p.lead;
    const int8_t* wrow = p.qw + c * 9;
    int wr[3];   // reversed filter rows: byte m = W[kh][2 - m], byte 3 zero
#pragma unroll
    for (int kh = 0; kh < 3; ++kh) {
        typedef int i1 __attribute__((ext_vector_type(1), aligned(1)));
        const int raw = (*reinterpret_cast<const i1*>(wrow + (p.flip ? 2 - kh : kh) * 3))[0];
        wr[kh] = (int)__builtin_amdgcn_perm(0u, (unsigned)raw, p.flip ? 0x0c020100u : 0x0c000102u);
    }
    int acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0;
#pragma unroll
    for (int k = 0; k < 6; ++k) {
        // gradient row h0 - 1 + k serves output row h0 + a through filter row kh = a + 2 - k
        const int r = min(h0 - 1 + k, p.Hin);
        unsigned lo, hi;
        load8(g, (int64_t)((int)n * p.img_rows + r) * p.row_pitch + (w0 - 1), lo, hi);
        const int win[4] = {(int)lo, (int)__builtin_amdgcn_alignbyte(hi, lo, 1), (int)__builtin_amdgcn_alignbyte(hi, lo, 2),
                            (int)__builtin_amdgcn_alignbyte(hi, lo, 3)};
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const int kh = a + 2 - k;
            if (kh < 0 || kh > 2) continue;
#pragma unroll
            for (int b = 0; b < 4; ++b) acc[a][b] = dot4(win[b], wr[kh], acc[a][b]);
        }
    }
    const float scale = (*p.s_w / 127.0f) * (p.s_g[p.per_chan ? c : 0] / 127.0f);
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int h = h0 + a;
        if (h >= p.Hin) break;
        const int64_t o = ((int64_t)nc * p.Hin + h) * p.Win + w0;
        store_result4(p.dX, o, (float)acc[a][0] * scale, (float)acc[a][1] * scale, (float)acc[a][2] * scale, (float)acc[a][3] * scale, p.bf16, p.nt);
        if (p.acc_out) *reinterpret_cast<int4*>(p.acc_out + o) = make_int4(acc[a][0], acc[a][1], acc[a][2], acc[a][3]);
    }
}

// Data gradient, 3 x 3, stride 2, padding 1, row length a multiple of four (MobileNetV2's strided layers): a thread
// produces a 4 x 4 block of outputs.  With h = 2a + i, w = 2b + j the live taps of an output depend only on the
// parities: (i, j) = (0, 0) reads g[a][b] W11;  (0, 1): g[a][b] W12 + g[a][b+1] W10;  (1, 0): g[a][b] W21 + g[a+1][b] W01;
// (1, 1): g[a][b] W22 + g[a][b+1] W20 + g[a+1][b] W02 + g[a+1][b+1] W00.  So the four outputs of a 2 x 2 block are four
// dot4 products of ONE dword - the gradient's 2 x 2 neighbourhood (g[a][b], g[a][b+1], g[a+1][b], g[a+1][b+1]) - with
// four weight dwords that are the same for every block of the channel.  The 4 x 4 outputs need three gradient rows of
// three bytes each: three loads, four byte permutes and sixteen dot4 in place of the sixteen-odd instructions per
// output of the row kernel above (which was bound by its instruction count, not by the result it writes).
// Rows past the gradient's last one are never needed for a stored output; their index is clamped to the zero row
// that follows every image.
__global__ __launch_bounds__(kBlock) void k_dwise_dx_s2_block(DxArgs p) {
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    const uint32_t rq = fdiv(i, p.div_wq);
    const int m = (int)(i - rq * (uint32_t)p.wq);
    const uint32_t nc = fdiv(rq, p.div_hq);
    if (nc >= (uint32_t)p.N * p.C) return;
    const int A = (int)(rq - nc * (uint32_t)p.hq);
    const uint32_t n = fdiv(nc, p.div_c);
    const int c = (int)(nc - n * (uint32_t)p.C);

    const int8_t* g = p.qg + (int64_t)c * p.chan_pitch + p.lead;
    // gradient rows 2A, 2A+1, 2A+2 from column 2m on: bytes 0..2 of R[k] are columns 2m..2m+2
    unsigned R[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        const int r = min(2 * A + k, p.Ho);
        const int64_t off = (int64_t)((int)n * p.img_rows + r) * p.row_pitch + 2 * m;
        const v2i_a4 d = *reinterpret_cast<const v2i_a4*>(g + (off & ~(int64_t)3));
        R[k] = __builtin_amdgcn_alignbyte((unsigned)d[1], (unsigned)d[0], (unsigned)(off & 3));
    }
    // weight dwords by output parity (byte t of the filter is W[t/3][t%3]; bytes past the ninth are not selected)
    unsigned wlo, whi;
    load8(p.qw, (int64_t)c * 9, wlo, whi);
    const unsigned w22 = (unsigned)(uint8_t)p.qw[c * 9 + 8];
    const int Wee = (int)__builtin_amdgcn_perm(whi, wlo, 0x0c0c0c04u);           // W11 . . .
    const int Weo = (int)__builtin_amdgcn_perm(whi, wlo, 0x0c0c0305u);           // W12 W10 . .
    const int Woe = (int)__builtin_amdgcn_perm(whi, wlo, 0x0c010c07u);           // W21 . W01 .
    const int Woo = (int)(__builtin_amdgcn_perm(whi, wlo, 0x0002060cu) | w22);   // W22 W20 W02 W00
    int acc[4][4];
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        // 2 x 2 neighbourhoods of the two blocks of row pair a: (g[a][b], g[a][b+1], g[a+1][b], g[a+1][b+1]), b = 0, 1
        const int P0 = (int)__builtin_amdgcn_perm(R[a + 1], R[a], 0x05040100u);
        const int P1 = (int)__builtin_amdgcn_perm(R[a + 1], R[a], 0x06050201u);
        acc[2 * a][0] = dot4(P0, Wee, 0);
        acc[2 * a][1] = dot4(P0, Weo, 0);
        acc[2 * a][2] = dot4(P1, Wee, 0);
        acc[2 * a][3] = dot4(P1, Weo, 0);
        acc[2 * a + 1][0] = dot4(P0, Woe, 0);
        acc[2 * a + 1][1] = dot4(P0, Woo, 0);
        acc[2 * a + 1][2] = dot4(P1, Woe, 0);
        acc[2 * a + 1][3] = dot4(P1, Woo, 0);
    }
    const float scale = (*p.s_w / 127.0f) * (p.s_g[p.per_chan ? c : 0] / 127.0f);
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const int h = 4 * A + rr;
        if (h >= p.Hin) break;
        const int64_t o = ((int64_t)nc * p.Hin + h) * p.Win + 4 * m;
        store_result4(p.dX, o, (float)acc[rr][0] * scale, (float)acc[rr][1] * scale, (float)acc[rr][2] * scale, (float)acc[rr][3] * scale, p.bf16, p.nt);
        if (p.acc_out) *reinterpret_cast<int4*>(p.acc_out + o) = make_int4(acc[rr][0], acc[rr][1], acc[rr][2], acc[rr][3]);
    }
}

// Data gradient, power-of-two stride, any dilation, extents up to 7: a thread produces four adjacent
// outputs; a tap contributes where (h + pad - kh*dil) and (w + pad - kw*dil) are multiples of the stride.
__global__ __launch_bounds__(kBlock) void k_dwise_dx_any(DxArgs p) {
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    const uint32_t rows = (uint32_t)p.N * p.C * p.Hin;
    const uint32_t row = fdiv(i, p.div_wq);
    if (row >= rows) return;
    const int w0 = 4 * (int)(i - row * (uint32_t)p.wq);
    const uint32_t nc = fdiv(row, p.div_h);
    const int h = (int)(row - nc * (uint32_t)p.Hin);
    const uint32_t n = fdiv(nc, p.div_c);
    const int c = (int)(nc - n * (uint32_t)p.C);

    const int8_t* g = p.qg + (int64_t)c * p.chan_pitch + p.lead;
    const int8_t* wf = p.qw + c * (p.kH * p.kW);
    const int smask = (1 << p.s_log2) - 1;
    int acc[4] = {0, 0, 0, 0};
    for (int kh = 0; kh < p.kH; ++kh) {
        const int th = h + p.pH - kh * p.dH;
        if (th & smask) continue;
        const int64_t rbase = (int64_t)((int)n * p.img_rows + (th >> p.s_log2)) * p.row_pitch;
        for (int kw = 0; kw < p.kW; ++kw) {
            const int wv = wf[kh * p.kW + kw];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int tw = w0 + j + p.pW - kw * p.dW;
                const bool ok = (tw & smask) == 0;
                const int8_t* src = ok ? g + (rbase + (tw >> p.s_log2)) : reinterpret_cast<const int8_t*>(g_zero64);
                acc[j] += (int)*src * wv;
            }
        }
    }
    const float scale = (*p.s_w / 127.0f) * (p.s_g[p.per_chan ? c : 0] / 127.0f);
    const int64_t o = (int64_t)row * p.Win + w0;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (w0 + j < p.Win) {
            store_result(p.dX, o + j, (float)acc[j] * scale, p.bf16);
            if (p.acc_out) p.acc_out[o + j] = acc[j];
        }
}

// ---------------------------------------------------------------------------------------------
// Filter gradient:  acc[c][t] = sum_f G[c][f] * X[c][tap_off[t] + f]  - per channel, T dot products
// over the flat axis (the same shifted correlation the dense kernel computes, with M = N = 1).
// Workgroup (c, slab) sweeps its part of the axis 4096 bytes at a time: a thread takes 16 aligned
// bytes of G and, for every tap, the 16 activation bytes at the tap's offset (byte aligned; the nine
// windows of a 3 x 3 filter overlap almost entirely, so they come from the same cache lines).
// Partial sums go to [c][slab][t]; k_dwise_dw_reduce adds the slabs and de-quantizes.
// ---------------------------------------------------------------------------------------------
constexpr int kDwTaps = 9;
struct DwiseDwArgs {
    const int8_t* g;
    const int8_t* x;
    int64_t g_chan_pitch, x_chan_pitch;
    int64_t klen;          // bytes of a gradient plane (multiple of 256)
    int64_t off[kDwTaps];  // unused slots repeat slot 0 (computed, never stored)
    int T, C, slabs;
    int32_t* part;         // [C][slabs][kDwTaps]
};

// ROWS3 >= 0: 3 x 3 filter at unit stride and dilation with row_pitch mod 4 == ROWS3 - the three windows of a filter
// row come out of one 24-byte fetch with compile-time shifts (7 loads per 16 positions instead of 19).
template <int ROWS3>
__global__ __launch_bounds__(kBlock) void k_dwise_dw(DwiseDwArgs p) {
    __shared__ int l_red[kBlock / kWave][kDwTaps];
    const int c = blockIdx.x / p.slabs, slab = blockIdx.x % p.slabs;
    const int tid = threadIdx.x;
    const int64_t iters_total = p.klen / kDwSlabBytes + ((p.klen % kDwSlabBytes) ? 1 : 0);
    const int64_t per = iters_total / p.slabs, rem = iters_total % p.slabs;
    const int64_t it0 = slab * per + std::min<int64_t>(slab, rem);
    const int64_t it1 = it0 + per + (slab < rem ? 1 : 0);
    const int8_t* g = p.g + (int64_t)c * p.g_chan_pitch;
    const int8_t* x = p.x + (int64_t)c * p.x_chan_pitch;

    int acc[kDwTaps];
#pragma unroll
    for (int t = 0; t < kDwTaps; ++t) acc[t] = 0;
    for (int64_t it = it0; it < it1; ++it) {
        const int64_t f = it * kDwSlabBytes + 16 * tid;
        const bool live = f < p.klen;   // klen is a multiple of 256, so a live thread has all 16 bytes
        const int64_t fc = live ? f : 0;
        v4i gv = *reinterpret_cast<const v4i*>(g + fc);
        if (!live) gv = v4i{0, 0, 0, 0};
        if (ROWS3 >= 0) {
#pragma unroll
            for (int kh = 0; kh < 3; ++kh) {
                const int r0 = (kh * ROWS3) & 3;   // byte shift of the row's first window; off[3*kh] = kh*row_pitch
                const int8_t* src = x + ((p.off[3 * kh] & ~(int64_t)3) + fc);
                const v4i_a4 lo = *reinterpret_cast<const v4i_a4*>(src);
                const v2i_a4 hi = *reinterpret_cast<const v2i_a4*>(src + 16);
                const unsigned d[6] = {(unsigned)lo[0], (unsigned)lo[1], (unsigned)lo[2], (unsigned)lo[3], (unsigned)hi[0], (unsigned)hi[1]};
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) {
                    const int sft = r0 + kw, j = sft >> 2, sh = sft & 3;
                    const int t = 3 * kh + kw;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int w = sh ? (int)__builtin_amdgcn_alignbyte(d[j + i + 1], d[j + i], (unsigned)sh) : (int)d[j + i];
                        acc[t] = dot4(gv[i], w, acc[t]);
                    }
                }
            }
        } else {
#pragma unroll
            for (int t = 0; t < kDwTaps; ++t) {
                // A byte-aligned 16-byte load runs at half the rate of a dword-aligned one here: fetch the 20 bytes from
                // the dword below the window and shift (the shift is the same for every thread: f is a multiple of 16).
                const int64_t o = p.off[t] + fc;
                const int8_t* src = x + (o & ~(int64_t)3);
                const unsigned sh = (unsigned)(p.off[t] & 3);
                const v4i_a4 lo = *reinterpret_cast<const v4i_a4*>(src);
                const int hi = *reinterpret_cast<const int*>(src + 16);
                const int w0 = (int)__builtin_amdgcn_alignbyte((unsigned)lo[1], (unsigned)lo[0], sh);
                const int w1 = (int)__builtin_amdgcn_alignbyte((unsigned)lo[2], (unsigned)lo[1], sh);
                const int w2 = (int)__builtin_amdgcn_alignbyte((unsigned)lo[3], (unsigned)lo[2], sh);
                const int w3 = (int)__builtin_amdgcn_alignbyte((unsigned)hi, (unsigned)lo[3], sh);
                acc[t] = dot4(gv[0], w0, acc[t]);
                acc[t] = dot4(gv[1], w1, acc[t]);
                acc[t] = dot4(gv[2], w2, acc[t]);
                acc[t] = dot4(gv[3], w3, acc[t]);
            }
        }
    }
#pragma unroll
    for (int t = 0; t < kDwTaps; ++t) {
        int v = acc[t];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o);
        if (tid % kWave == 0) l_red[tid / kWave][t] = v;
    }
    __syncthreads();
    if (tid < kDwTaps)
        p.part[((int64_t)c * p.slabs + slab) * kDwTaps + tid] = l_red[0][tid] + l_red[1][tid] + l_red[2][tid] + l_red[3][tid];
}

// One wave per filter element: its lanes take the slabs (independent loads, all in flight), then a shuffle tree.
__global__ __launch_bounds__(kBlock) void k_dwise_dw_reduce(const int32_t* __restrict__ part, int C, int slabs, int T,
                                                            const float* s_x, const float* __restrict__ s_chan,
                                                            float* __restrict__ dW, int32_t* __restrict__ acc_out, int bf16) {
    const int lane = threadIdx.x % kWave;
    const int i = blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;   // filter element (c, t)
    if (i >= C * T) return;
    const int c = i / T, t = i % T;
    int a = 0;
    for (int s = lane; s < slabs; s += kWave) a += part[((int64_t)c * slabs + s) * kDwTaps + t];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) a += __shfl_down(a, o);
    if (lane != 0) return;
    store_result(dW, i, (float)a * ((*s_x / 127.0f) * (s_chan[c] / 127.0f)), bf16);
    if (acc_out) acc_out[i] = a;
}

int log2_exact(int v) {
    int l = 0;
    while ((1 << l) < v) ++l;
    return (1 << l) == v ? l : -1;
}

int dw_slabs(const daq_conv_desc& d, int64_t klen) {
    const int64_t iters = ceil_div(klen, kDwSlabBytes);
    int64_t s = ceil_div(2048, d.Cout);
    if (s > iters) s = iters;
    if (s > 256) s = 256;
    return (int)std::max<int64_t>(1, s);
}

}  // namespace

bool depthwise_dx_supported(const daq_conv_desc& d) {
    if (!is_depthwise(d) || d.strideH != d.strideW || log2_exact(d.strideH) < 0) return false;
    if (d.kH > kMaxK || d.kW > kMaxK) return false;
    return (int64_t)d.N * d.Cin * d.Hin * ceil_div(d.Win, 4) < ((int64_t)1 << 31);
}

// Forward pass, 3 x 3, stride 2, padding 1, on the channel-major activation planes (one plane per parity of the padded
// row and column, so a tap is a unit-stride read): tap (kh, kw) of output (ho, wo) is element (ho + kh/2, wo + kw/2)
// of plane (kh % 2, kw % 2).  A thread produces four adjacent outputs of a row from six 8-byte fetches (two rows of
// planes (0, 0) and (0, 1), one row of (1, 0) and (1, 1)); which byte a tap reads is the same for every thread.
struct FwdS2Args {
    const int8_t* qx;      // [C][4 planes][plane_pitch]
    const int8_t* qw;      // plain filter copy, [C][9]
    int64_t chan_pitch, plane_pitch;
    int lead, img_rows, row_pitch;
    int N, C, Ho, Wo, wq;
    FastDiv div_wq, div_ho, div_c;
    const float* s_x;
    const float* s_w;
    float* Y;
    int32_t* acc_out;
};

__global__ __launch_bounds__(kBlock) void k_dwise_fwd_s2(FwdS2Args p) {
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    const uint32_t row = fdiv(i, p.div_wq);
    if (row >= (uint32_t)p.N * p.C * p.Ho) return;
    const int wo0 = 4 * (int)(i - row * (uint32_t)p.wq);
    const uint32_t nc = fdiv(row, p.div_ho);
    const int ho = (int)(row - nc * (uint32_t)p.Ho);
    const uint32_t n = fdiv(nc, p.div_c);
    const int c = (int)(nc - n * (uint32_t)p.C);
    const int8_t* x = p.qx + (int64_t)c * p.chan_pitch + p.lead;
    const int8_t* wf = p.qw + c * 9;
    const int64_t at = (int64_t)((int)n * p.img_rows + ho) * p.row_pitch + wo0;
    int acc[4] = {0, 0, 0, 0};
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int pw = 0; pw < 2; ++pw) {
            // plane (kh % 2, pw), row ho + kh / 2: serves kw = pw (column shift 0) and, for pw = 0, kw = 2 (shift 1)
            unsigned lo, hi;
            load8(x + (int64_t)((kh & 1) * 2 + pw) * p.plane_pitch, at + (int64_t)(kh >> 1) * p.row_pitch, lo, hi);
            const int w_a = wf[kh * 3 + pw];
            const int w_b = pw == 0 ? wf[kh * 3 + 2] : 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                acc[j] += __builtin_amdgcn_sbfe((int)lo, 8 * j, 8) * w_a;
                if (pw == 0) acc[j] += __builtin_amdgcn_sbfe((int)(j < 3 ? lo : hi), 8 * ((j + 1) & 3), 8) * w_b;
            }
        }
    const float scale = (*p.s_x / 127.0f) * (*p.s_w / 127.0f);
    const int64_t o = (int64_t)row * p.Wo + wo0;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (wo0 + j < p.Wo) {
            p.Y[o + j] = (float)acc[j] * scale;
            if (p.acc_out) p.acc_out[o + j] = acc[j];
        }
}

// Forward pass of the 3 x 3, unit-stride, padding-1 depthwise layers: the data-gradient kernels on the channel-major
// activation planes, with the filter rotated by 180 degrees (4 x 4 output blocks where rows are a multiple of four,
// four outputs of a row per thread otherwise).
bool depthwise_fwd_supported(const daq_conv_desc& d) {
    return is_depthwise(d) && d.kH == 3 && d.kW == 3 && d.strideH == d.strideW && (d.strideH == 1 || d.strideH == 2) &&
           d.dilH == 1 && d.dilW == 1 && d.padH == 1 && d.padW == 1 &&
           (int64_t)d.N * d.Cin * d.Hin * ceil_div(d.Win, 4) < ((int64_t)1 << 31);
}

daq_status conv_fwd_depthwise(const daq_conv_desc& d, const int8_t* qx_cnhw, const int8_t* qw, const float* s_x,
                              const float* s_w, float* Y, int32_t* acc, hipStream_t st) {
    daq_layout Lx;
    daq_wpack_layout Lw;
    if (daq_layout_qx_cnhw(&d, &Lx) != DAQ_OK || daq_layout_qw(&d, &Lw) != DAQ_OK) return DAQ_ERR_INVALID_ARG;
    if (d.strideH == 2) {
        if (Lx.phases_h != 2 || Lx.phases_w != 2) return DAQ_ERR_INVALID_ARG;
        FwdS2Args f{};
        f.qx = qx_cnhw;
        f.qw = qw + Lw.off_plain;
        f.chan_pitch = Lx.chan_pitch; f.plane_pitch = Lx.plane_pitch;
        f.lead = (int)Lx.lead; f.img_rows = Lx.img_rows; f.row_pitch = Lx.row_pitch;
        f.N = d.N; f.C = d.Cin; f.Ho = daq_out_h(&d); f.Wo = daq_out_w(&d);
        f.wq = (int)ceil_div(f.Wo, 4);
        f.div_wq = make_fastdiv((uint32_t)f.wq);
        f.div_ho = make_fastdiv((uint32_t)f.Ho);
        f.div_c = make_fastdiv((uint32_t)d.Cin);
        f.s_x = s_x; f.s_w = s_w; f.Y = Y; f.acc_out = acc;
        const int64_t threads = (int64_t)d.N * d.Cin * f.Ho * f.wq;
        DAQ_LAUNCH("conv_fwd_depthwise", st,
                   hipLaunchKernelGGL(k_dwise_fwd_s2, dim3((unsigned)ceil_div(threads, kBlock)), dim3(kBlock), 0, st, f));
        return DAQ_OK;
    }
    if (Lx.phases_h != 1 || Lx.phases_w != 1) return DAQ_ERR_INVALID_ARG;
    DxArgs a{};
    a.qg = qx_cnhw;
    a.qw = qw + Lw.off_plain;
    a.chan_pitch = Lx.chan_pitch;
    a.lead = (int)Lx.lead; a.img_rows = Lx.img_rows; a.row_pitch = Lx.row_pitch;
    a.N = d.N; a.C = d.Cin; a.Hin = d.Hin; a.Win = d.Win;   // the result has the input's extent
    a.kH = 3; a.kW = 3; a.pH = 1; a.pW = 1; a.dH = 1; a.dW = 1;
    a.wq = (int)ceil_div(d.Win, 4);
    a.hq = (int)ceil_div(d.Hin, 4);
    a.div_wq = make_fastdiv((uint32_t)a.wq);
    a.div_hq = make_fastdiv((uint32_t)a.hq);
    a.div_h = make_fastdiv((uint32_t)d.Hin);
    a.div_c = make_fastdiv((uint32_t)d.Cin);
    a.Ho = d.Hin;
    a.s_g = s_x; a.s_w = s_w; a.dX = Y; a.acc_out = acc;
    a.flip = 1;
    a.nt = (int64_t)d.N * d.Cin * d.Hin * d.Win * 4 >= kStreamBytes;
    if (d.Win % 4 == 0) {
        const int64_t blocks4 = (int64_t)d.N * d.Cin * a.hq * a.wq;
        DAQ_LAUNCH("conv_fwd_depthwise", st,
                   hipLaunchKernelGGL(k_dwise_dx_unit_block, dim3((unsigned)ceil_div(blocks4, kBlock)), dim3(kBlock), 0, st, a));
    } else {
        const int64_t threads = (int64_t)d.N * d.Cin * d.Hin * a.wq;
        DAQ_LAUNCH("conv_fwd_depthwise", st,
                   hipLaunchKernelGGL((k_dwise_dx_unit<3, 3>), dim3((unsigned)ceil_div(threads, kBlock)), dim3(kBlock), 0, st, a));
    }
    return DAQ_OK;
}

daq_status conv_bwd_data_depthwise(const daq_conv_desc& d, const int8_t* qg, const float* s_g, const int8_t* qw,
                                   const float* s_w, float* dX, int32_t* acc, hipStream_t st, bool per_channel, bool bf16) {
    daq_layout Lg;
    daq_wpack_layout Lw;
    if (daq_layout_qg(&d, &Lg) != DAQ_OK || daq_layout_qw(&d, &Lw) != DAQ_OK || Lg.kind != DAQ_LAYOUT_CNHW)
        return DAQ_ERR_INVALID_ARG;
    DxArgs a{};
    a.qg = qg;
    a.qw = qw + Lw.off_plain;
    a.chan_pitch = Lg.chan_pitch;
    a.lead = (int)Lg.lead; a.img_rows = Lg.img_rows; a.row_pitch = Lg.row_pitch;
    a.N = d.N; a.C = d.Cin; a.Hin = d.Hin; a.Win = d.Win;
    a.kH = d.kH; a.kW = d.kW; a.pH = d.padH; a.pW = d.padW; a.dH = d.dilH; a.dW = d.dilW;
    a.s_log2 = log2_exact(d.strideH);
    a.wq = (int)ceil_div(d.Win, 4);
    a.div_wq = make_fastdiv((uint32_t)a.wq);
    a.div_h = make_fastdiv((uint32_t)d.Hin);
    a.div_c = make_fastdiv((uint32_t)d.Cin);
    a.s_g = s_g; a.s_w = s_w; a.dX = dX; a.acc_out = acc;
    a.per_chan = per_channel ? 1 : 0;
    a.bf16 = bf16 ? 1 : 0;
    a.nt = (int64_t)d.N * d.Cin * d.Hin * d.Win * (bf16 ? 2 : 4) >= kStreamBytes;
    const int64_t threads = (int64_t)d.N * d.Cin * d.Hin * a.wq;
    const dim3 grid((unsigned)ceil_div(threads, kBlock));
    const bool unit = d.strideH == 1 && d.dilH == 1 && d.dilW == 1 && d.kW <= 4;
    // strided form: the columns four outputs can read, (3 + kW - 1) / stride + 1 of them, must fit the 8-byte load
    const bool strided = d.strideH > 1 && d.dilH == 1 && d.dilW == 1 && (3 + d.kW - 1) / d.strideH + 2 <= 8;
    const bool k33 = d.kH == 3 && d.kW == 3;
    const bool block_s2 = strided && k33 && d.strideH == 2 && d.padH == 1 && d.padW == 1 && d.Win % 4 == 0;
    const bool block_s1 = unit && k33 && d.padH == 1 && d.padW == 1 && d.Win % 4 == 0;
    if (block_s2 || block_s1) {
        a.hq = (int)ceil_div(d.Hin, 4);
        a.div_hq = make_fastdiv((uint32_t)a.hq);
        a.Ho = daq_out_h(&d);
        const int64_t blocks4 = (int64_t)d.N * d.Cin * a.hq * a.wq;   // fewer than `threads`, which the caller bounded
        const dim3 bgrid((unsigned)ceil_div(blocks4, kBlock));
        if (block_s2)
            DAQ_LAUNCH("conv_bwd_data_depthwise", st, hipLaunchKernelGGL(k_dwise_dx_s2_block, bgrid, dim3(kBlock), 0, st, a));
        else
            DAQ_LAUNCH("conv_bwd_data_depthwise", st, hipLaunchKernelGGL(k_dwise_dx_unit_block, bgrid, dim3(kBlock), 0, st, a));
        return DAQ_OK;
    }
    if (unit && k33)
        DAQ_LAUNCH("conv_bwd_data_depthwise", st, hipLaunchKernelGGL((k_dwise_dx_unit<3, 3>), grid, dim3(kBlock), 0, st, a));
    else if (unit)
        DAQ_LAUNCH("conv_bwd_data_depthwise", st, hipLaunchKernelGGL((k_dwise_dx_unit<0, 0>), grid, dim3(kBlock), 0, st, a));
    else if (strided && k33 && d.strideH == 2 && d.padH == 1 && d.padW == 1)
        DAQ_LAUNCH("conv_bwd_data_depthwise", st,
                   hipLaunchKernelGGL((k_dwise_dx_strided<3, 3, 1, 1>), grid, dim3(kBlock), 0, st, a));
    else if (strided && k33)
        DAQ_LAUNCH("conv_bwd_data_depthwise", st,
                   hipLaunchKernelGGL((k_dwise_dx_strided<3, 3, -1, -1>), grid, dim3(kBlock), 0, st, a));
    else if (strided)
        DAQ_LAUNCH("conv_bwd_data_depthwise", st,
                   hipLaunchKernelGGL((k_dwise_dx_strided<0, 0, -1, -1>), grid, dim3(kBlock), 0, st, a));
    else
        DAQ_LAUNCH("conv_bwd_data_depthwise", st, hipLaunchKernelGGL(k_dwise_dx_any, grid, dim3(kBlock), 0, st, a));
    return DAQ_OK;
}

bool depthwise_dw_supported(const daq_conv_desc& d) { return is_depthwise(d) && d.kH * d.kW <= kDwTaps; }

size_t depthwise_dw_ws_bytes(const daq_conv_desc& d) {
    daq_layout Lg;
    if (!depthwise_dw_supported(d) || daq_layout_vq(&d, &Lg) != DAQ_OK) return 0;
    return (size_t)round_up((int64_t)d.Cout * dw_slabs(d, Lg.plane_pitch) * kDwTaps * 4, 256);
}

daq_status conv_bwd_filter_depthwise(const daq_conv_desc& d, const int8_t* qx, const float* s_x, const int8_t* vq,
                                     const float* s_chan, float* dW, int32_t* acc, void* ws, hipStream_t st, bool bf16) {
    daq_layout Lx, Lg;
    if (daq_layout_qx_cnhw(&d, &Lx) != DAQ_OK || daq_layout_vq(&d, &Lg) != DAQ_OK) return DAQ_ERR_INVALID_ARG;
    DwiseDwArgs a{};
    a.g = vq;
    a.x = qx;
    a.g_chan_pitch = Lg.chan_pitch;
    a.x_chan_pitch = Lx.chan_pitch;
    a.klen = Lg.plane_pitch;
    a.T = d.kH * d.kW;
    a.C = d.Cout;
    a.slabs = dw_slabs(d, Lg.plane_pitch);
    a.part = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(ws) + 256);
    // window start of every tap inside an activation channel (stride-phase plane + shift), as in the dense kernel
    for (int t = 0; t < kDwTaps; ++t) a.off[t] = 0;
    for (int kh = 0; kh < d.kH; ++kh)
        for (int kw = 0; kw < d.kW; ++kw) {
            const int ph = (kh * d.dilH) % Lx.phases_h, pw = (kw * d.dilW) % Lx.phases_w;
            a.off[kh * d.kW + kw] = (int64_t)(ph * Lx.phases_w + pw) * Lx.plane_pitch +
                                    (int64_t)(kh * d.dilH / Lx.phases_h) * Lx.row_pitch + (kw * d.dilW / Lx.phases_w);
        }
    for (int t = a.T; t < kDwTaps; ++t) a.off[t] = a.off[0];
    const dim3 grid((unsigned)(d.Cout * a.slabs));
    const bool rows3 = d.kH == 3 && d.kW == 3 && Lx.phases_h == 1 && Lx.phases_w == 1 && d.dilH == 1 && d.dilW == 1;
    const int q4 = rows3 ? (Lx.row_pitch & 3) : -1;
    if (q4 == 0) DAQ_LAUNCH("conv_bwd_filter_depthwise", st, hipLaunchKernelGGL(k_dwise_dw<0>, grid, dim3(kBlock), 0, st, a));
    else if (q4 == 1) DAQ_LAUNCH("conv_bwd_filter_depthwise", st, hipLaunchKernelGGL(k_dwise_dw<1>, grid, dim3(kBlock), 0, st, a));
    else if (q4 == 2) DAQ_LAUNCH("conv_bwd_filter_depthwise", st, hipLaunchKernelGGL(k_dwise_dw<2>, grid, dim3(kBlock), 0, st, a));
    else if (q4 == 3) DAQ_LAUNCH("conv_bwd_filter_depthwise", st, hipLaunchKernelGGL(k_dwise_dw<3>, grid, dim3(kBlock), 0, st, a));
    else DAQ_LAUNCH("conv_bwd_filter_depthwise", st, hipLaunchKernelGGL(k_dwise_dw<-1>, grid, dim3(kBlock), 0, st, a));
    DAQ_LAUNCH("dw_reduce", st,
               hipLaunchKernelGGL(k_dwise_dw_reduce, dim3((unsigned)ceil_div(d.Cout * a.T, kBlock / kWave)), dim3(kBlock), 0, st,
                                  a.part, d.Cout, a.slabs, a.T, s_x, s_chan, dW, acc, bf16 ? 1 : 0));
    return DAQ_OK;
}

}  // namespace daq
