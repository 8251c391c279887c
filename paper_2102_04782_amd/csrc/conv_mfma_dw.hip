// Filter gradient  q(G_W) = q(X') (x) vq(G')  on the gfx950 int8 matrix cores.
//
// Both operands are channel-major (the paper's dimension transformation), with images in pitched
// slots that carry the zero padding.  With f the flattened (n, row, col) position of a gradient
// element, the activation element that filter tap (kh, kw) pairs with it sits at f + kh*row_pitch + kw
// of the activation plane (unit stride, unit dilation).  The product is therefore a set of shifted
// correlations over one flat axis:
//
//     acc[co][ci][kh][kw] = sum_f  G[co][f] * X[ci][f + kh*row_pitch + kw]
//
// i.e. a GEMM with M = Cout, N = Cin*kH*kW, K = the flat axis, whose B operand is the same bytes
// read at kH*kW offsets.  v_mfma_i32_16x16x64_i8 wants 16 consecutive K bytes per lane: for G they
// are an aligned 16-byte LDS read; for X they start at an arbitrary byte, so a lane reads the six
// dwords that cover the three kw windows of one kh once and realigns with v_alignbyte_b32.
//
// Workgroup = 4 waves.  A wave owns a 64 (co) x 16 (ci) x kH*kW accumulator tile (144 VGPRs for
// 3x3).  The four waves either take four ci blocks (WGK = 1) or share one ci block and split the
// K steps of every staged chunk (WGK = 4, reduced through LDS at the end); the latter keeps all 256
// CUs busy on layers with few channels.  K is also split across workgroups; partial tiles are
// combined with int32 atomics (exact, order independent) and de-quantized by a small epilogue.
#include "daq_internal.h"

namespace daq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kKC = 256;          // K bytes staged per chunk (4 MFMA K-steps of 64)
constexpr int kPA = kKC + 16;     // LDS row pitch of the G tile: +16 B rotates banks between rows
constexpr int kBM = 64;           // co rows per workgroup

struct DwArgs {
    const int8_t* g;      // vq, [Cout][klen]
    const int8_t* x;      // q(X'), [Cin][chan_pitch_x]
    int64_t klen;         // bytes of the flat axis (multiple of 256)
    int64_t x_chan_pitch;
    int Cout, Cin;
    int row_pitch;        // Wq
    int pb;               // LDS row pitch of the X tile (bytes, multiple of 16)
    int nchunks;          // klen / kKC
    int splits;           // workgroups along K
    int tiles_n;          // ci tiles
    int32_t* ws;          // int32 accumulators [Cout][Cin][kH*kW], zeroed beforehand (splits > 1 only)
    // splits == 1: the tile is complete, de-quantize and store it directly
    const float* s_x;
    const float* s_chan;
    float* dW;
    int32_t* acc_out;
};

__device__ __forceinline__ int alignbyte(int hi, int lo, int sh) {
    return (int)__builtin_amdgcn_alignbyte((unsigned)hi, (unsigned)lo, (unsigned)sh);
}

template <int KH, int KW, int WQ4, int WGK>
__global__ __launch_bounds__(256) void k_dw_mfma(DwArgs p) {
    constexpr int WGN = 4 / WGK;         // waves along ci
    constexpr int BN = 16 * WGN;         // ci rows per workgroup
    constexpr int T = KH * KW;
    extern __shared__ __align__(16) int8_t lds[];

    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int wn = wave % WGN, wk = wave / WGN;
    const int li = lane & 15, lg = lane >> 4;

    int b = blockIdx.x;
    const int split = b % p.splits; b /= p.splits;
    const int tn = b % p.tiles_n;
    const int tm = b / p.tiles_n;
    const int co0 = tm * kBM, ci0 = tn * BN;
    // chunks [c_begin, c_end) of this split
    const int per = p.nchunks / p.splits, rem = p.nchunks % p.splits;
    const int c_begin = split * per + min(split, rem);
    const int c_end = c_begin + per + (split < rem ? 1 : 0);

    const int a_bytes = kBM * kPA;
    const int b_bytes = BN * p.pb;
    const int stage_bytes = a_bytes + b_bytes;
    const int ub = p.pb / 16;            // 16-byte units per X row
    const int a_units = kBM * (kKC / 16);
    const int b_units = BN * ub;
    constexpr int A_PER_T = kBM * (kKC / 16) / 256;  // 4
    const int b_per_t = (b_units + 255) / 256;

    v4i acc[4][T];
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int t = 0; t < T; ++t) acc[m][t] = v4i{0, 0, 0, 0};

    // ---- staging helpers (global -> registers -> LDS) ----
    constexpr int MAXB = 12;             // enough for pb <= 768 with BN = 64
    uint4 ra[A_PER_T];
    uint4 rb[MAXB];
    auto load_chunk = [&](int chunk) {
        const int64_t k0 = (int64_t)chunk * kKC;
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i) {
            const int u = tid + 256 * i;
            const int row = u / (kKC / 16), c16 = u % (kKC / 16);
            const int co = co0 + row;
            ra[i] = (co < p.Cout) ? *reinterpret_cast<const uint4*>(p.g + (int64_t)co * p.klen + k0 + 16 * c16)
                                  : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < MAXB; ++i) {
            if (i < b_per_t) {
                const int u = tid + 256 * i;
                const int row = u / ub, c16 = u - row * ub;
                const int ci = ci0 + row;
                rb[i] = (u < b_units && ci < p.Cin)
                            ? *reinterpret_cast<const uint4*>(p.x + (int64_t)ci * p.x_chan_pitch + k0 + 16 * c16)
                            : make_uint4(0, 0, 0, 0);
            }
        }
    };
    auto store_chunk = [&](int buf) {
        int8_t* A = lds + buf * stage_bytes;
        int8_t* B = A + a_bytes;
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i) {
            const int u = tid + 256 * i;
            const int row = u / (kKC / 16), c16 = u % (kKC / 16);
            *reinterpret_cast<uint4*>(A + row * kPA + 16 * c16) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < MAXB; ++i) {
            if (i < b_per_t) {
                const int u = tid + 256 * i;
                if (u < b_units) {
                    const int row = u / ub, c16 = u - row * ub;
                    *reinterpret_cast<uint4*>(B + row * p.pb + 16 * c16) = rb[i];
                }
            }
        }
    };

    if (c_begin < c_end) {
        load_chunk(c_begin);
        store_chunk(0);
    }
    __syncthreads();

    for (int chunk = c_begin; chunk < c_end; ++chunk) {
        const int buf = (chunk - c_begin) & 1;
        const bool more = chunk + 1 < c_end;
        if (more) load_chunk(chunk + 1);

        const int8_t* A = lds + buf * stage_bytes;
        const int8_t* B = A + a_bytes + (wn * 16 + li) * p.pb;
#pragma unroll
        for (int ks = wk; ks < kKC / 64; ks += WGK) {
            v4i a[4];
#pragma unroll
            for (int m = 0; m < 4; ++m)
                a[m] = *reinterpret_cast<const v4i*>(A + (16 * m + li) * kPA + ks * 64 + 16 * lg);
#pragma unroll
            for (int kh = 0; kh < KH; ++kh) {
                constexpr int dummy = 0;
                (void)dummy;
                const int r0 = (kh * WQ4) & 3;  // (kh*row_pitch) mod 4, known at compile time
                const int byte0 = ks * 64 + 16 * lg + kh * p.row_pitch;
                const int* src = reinterpret_cast<const int*>(B + (byte0 - r0));
                int d[6];
#pragma unroll
                for (int i = 0; i < 6; ++i) d[i] = src[i];
#pragma unroll
                for (int kw = 0; kw < KW; ++kw) {
                    const int s = r0 + kw;
                    const int j = s >> 2, sh = s & 3;
                    v4i bf;
                    if (sh == 0) {
                        bf = v4i{d[j], d[j + 1], d[j + 2], d[j + 3]};
                    } else {
                        bf = v4i{alignbyte(d[j + 1], d[j], sh), alignbyte(d[j + 2], d[j + 1], sh),
                                 alignbyte(d[j + 3], d[j + 2], sh), alignbyte(d[j + 4], d[j + 3], sh)};
                    }
#pragma unroll
                    for (int m = 0; m < 4; ++m)
                        acc[m][kh * KW + kw] =
                            __builtin_amdgcn_mfma_i32_16x16x64_i8(a[m], bf, acc[m][kh * KW + kw], 0, 0, 0);
                }
            }
        }
        if (more) store_chunk(buf ^ 1);
        __syncthreads();
    }

    // ---- reduce the WGK waves that share a tile (through LDS, one wave at a time) ----
    if (WGK > 1) {
        int* red = reinterpret_cast<int*>(lds);
        for (int w = 1; w < WGK; ++w) {
            __syncthreads();
            if (wk == w) {
#pragma unroll
                for (int m = 0; m < 4; ++m)
#pragma unroll
                    for (int t = 0; t < T; ++t)
#pragma unroll
                        for (int r = 0; r < 4; ++r) red[((m * T + t) * 4 + r) * kWave + lane] = acc[m][t][r];
            }
            __syncthreads();
            if (wk == 0) {
#pragma unroll
                for (int m = 0; m < 4; ++m)
#pragma unroll
                    for (int t = 0; t < T; ++t)
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[m][t][r] += red[((m * T + t) * 4 + r) * kWave + lane];
            }
        }
        if (wk != 0) return;
    }

    // ---- a complete tile is de-quantized here; a partial one is added into the int32 accumulators ----
    const int ci = ci0 + wn * 16 + li;
    if (ci >= p.Cin) return;
    const bool direct = (p.splits == 1);
    const float sx = direct ? (*p.s_x / 127.0f) : 0.0f;
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int co = co0 + 16 * m + 4 * lg + r;
            if (co < p.Cout) {
                const int64_t off = ((int64_t)co * p.Cin + ci) * T;
                if (direct) {
                    const float sc = sx * (p.s_chan[co] / 127.0f);
#pragma unroll
                    for (int t = 0; t < T; ++t) {
                        p.dW[off + t] = (float)acc[m][t][r] * sc;
                        if (p.acc_out) p.acc_out[off + t] = acc[m][t][r];
                    }
                } else {
#pragma unroll
                    for (int t = 0; t < T; ++t) atomicAdd(p.ws + off + t, acc[m][t][r]);
                }
            }
        }
}

__global__ __launch_bounds__(256) void k_zero_i32(int32_t* p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0;
}

// dW[co][...] = acc * ((s_x/127) * (s_chan[co]/127))
__global__ __launch_bounds__(256) void k_dw_epilogue(const int32_t* __restrict__ ws, int64_t n, int per_co,
                                                     const float* s_x, const float* __restrict__ s_chan,
                                                     float* __restrict__ dW, int32_t* __restrict__ acc_out) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int co = (int)(i / per_co);
    const int32_t a = ws[i];
    dW[i] = (float)a * ((*s_x / 127.0f) * (s_chan[co] / 127.0f));
    if (acc_out) acc_out[i] = a;
}

struct Plan {
    bool ok;
    int wgk, splits, tiles_m, tiles_n, pb, nchunks;
    size_t lds_bytes;
};

Plan make_plan(const daq_conv_desc& d) {
    Plan pl{};
    pl.ok = false;
    if (d.groups != 1 || d.strideH != 1 || d.strideW != 1 || d.dilH != 1 || d.dilW != 1) return pl;
    if (!((d.kH == 3 && d.kW == 3) || (d.kH == 1 && d.kW == 1))) return pl;
    if (d.kH == 1 && (d.padH != 0 || d.padW != 0)) return pl;
    daq_layout Lx, Lg;
    if (daq_layout_qx_cnhw(&d, &Lx) != DAQ_OK || daq_layout_vq(&d, &Lg) != DAQ_OK) return pl;
    const int halo = (d.kH - 1) * Lx.row_pitch + (d.kW - 1) + 3 + 8;  // +3 realignment, +8: six dwords are read
    pl.pb = (int)round_up(kKC + halo, 16) + 16;
    pl.nchunks = (int)(Lg.plane_pitch / kKC);
    pl.tiles_m = (int)ceil_div(d.Cout, kBM);
    const int T = d.kH * d.kW;
    const int64_t outs = (int64_t)d.Cout * d.Cin * T;
    // Prefer a shape with enough output tiles to fill the 256 CUs without splitting K (no atomics, one
    // launch).  With few channels the four waves of a workgroup split K instead of ci, and K is also
    // split across workgroups, bounded by the atomic traffic it causes.
    const int64_t tiles1 = (int64_t)pl.tiles_m * ceil_div(d.Cin, 64);
    const int64_t tiles4 = (int64_t)pl.tiles_m * ceil_div(d.Cin, 16);
    int64_t s = 1;
    if (tiles1 >= 192) {
        pl.wgk = 1;
    } else {
        pl.wgk = 4;
        if (tiles4 < 192) {
            s = ceil_div(384, tiles4);
            const int64_t max_by_chunks = pl.nchunks / 2 > 0 ? pl.nchunks / 2 : 1;
            if (s > max_by_chunks) s = max_by_chunks;
            const int64_t max_by_atomics = (int64_t)4e6 / (outs > 0 ? outs : 1);
            if (s > max_by_atomics) s = max_by_atomics;
            if (s < 1) s = 1;
        }
    }
    const int bn = 16 * (4 / pl.wgk);
    pl.tiles_n = (int)ceil_div(d.Cin, bn);
    pl.splits = (int)s;
    const size_t stage = (size_t)kBM * kPA + (size_t)bn * pl.pb;
    pl.lds_bytes = 2 * stage;
    const size_t red = (size_t)4 * T * 4 * kWave * 4;
    if (pl.wgk > 1 && pl.lds_bytes < red) pl.lds_bytes = red;
    const int b_units = bn * (pl.pb / 16);
    if (pl.lds_bytes > 160 * 1024 || (b_units + 255) / 256 > 12) return pl;
    pl.ok = true;
    return pl;
}

template <int KH, int KW>
daq_status launch_dw(const Plan& pl, const DwArgs& a, int wq4, hipStream_t st) {
    const dim3 grid((unsigned)(pl.tiles_m * pl.tiles_n * pl.splits));
#define DAQ_DW_CASE(Q, K)                                                                                         \
    if (wq4 == Q && pl.wgk == K) {                                                                                \
        auto kern = k_dw_mfma<KH, KW, Q, K>;                                                                      \
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,                    \
                                (int)pl.lds_bytes) != hipSuccess)                                                 \
            return DAQ_ERR_HIP;                                                                                   \
        DAQ_LAUNCH("conv_bwd_filter_mfma", st, hipLaunchKernelGGL(kern, grid, dim3(256), pl.lds_bytes, st, a));   \
        return DAQ_OK;                                                                                            \
    }
    DAQ_DW_CASE(0, 1) DAQ_DW_CASE(1, 1) DAQ_DW_CASE(2, 1) DAQ_DW_CASE(3, 1)
    DAQ_DW_CASE(0, 4) DAQ_DW_CASE(1, 4) DAQ_DW_CASE(2, 4) DAQ_DW_CASE(3, 4)
#undef DAQ_DW_CASE
    return DAQ_ERR_UNSUPPORTED;
}

}  // namespace

bool bwd_filter_mfma_supported(const daq_conv_desc& d) { return make_plan(d).ok; }

size_t bwd_filter_mfma_ws_bytes(const daq_conv_desc& d) {
    return (size_t)round_up((int64_t)d.Cout * (d.Cin / d.groups) * d.kH * d.kW * 4, 256);
}

daq_status conv_bwd_filter_mfma(const daq_conv_desc& d, const int8_t* qx, const float* s_x, const int8_t* vq,
                                const float* s_chan, float* dW, int32_t* acc, void* ws, hipStream_t st) {
    const Plan pl = make_plan(d);
    if (!pl.ok) return DAQ_ERR_UNSUPPORTED;
    daq_layout Lx, Lg;
    if (daq_layout_qx_cnhw(&d, &Lx) != DAQ_OK || daq_layout_vq(&d, &Lg) != DAQ_OK) return DAQ_ERR_INVALID_ARG;
    const int T = d.kH * d.kW;
    const int64_t n = (int64_t)d.Cout * d.Cin * T;
    int32_t* wsi = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(ws) + 256);
    if (pl.splits > 1)
        DAQ_LAUNCH("zero_acc", st,
                   hipLaunchKernelGGL(k_zero_i32, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, st, wsi, n));
    DwArgs a{};
    a.g = vq;
    a.x = qx;
    a.klen = Lg.plane_pitch;
    a.x_chan_pitch = Lx.chan_pitch;
    a.Cout = d.Cout;
    a.Cin = d.Cin;
    a.row_pitch = Lx.row_pitch;
    a.pb = pl.pb;
    a.nchunks = pl.nchunks;
    a.splits = pl.splits;
    a.tiles_n = pl.tiles_n;
    a.ws = wsi;
    a.s_x = s_x;
    a.s_chan = s_chan;
    a.dW = dW;
    a.acc_out = acc;
    daq_status rc;
    if (d.kH == 3) rc = launch_dw<3, 3>(pl, a, Lx.row_pitch & 3, st);
    else rc = launch_dw<1, 1>(pl, a, 0, st);
    if (rc != DAQ_OK) return rc;
    if (pl.splits > 1)
        DAQ_LAUNCH("dw_epilogue", st,
               hipLaunchKernelGGL(k_dw_epilogue, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, st, wsi, n,
                                  d.Cin * T, s_x, s_chan, dW, acc));
    return DAQ_OK;
}

}  // namespace daq
