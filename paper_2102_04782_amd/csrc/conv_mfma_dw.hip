// Filter gradient  q(G_W) = q(X') (x) vq(G')  on the gfx950 int8 matrix cores: the general tap-table kernel (any
// stride, dilation, extent) and the 3 x 3 forms that serve rows too long for the LDS window of conv_mfma_dw32.hip.
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
// read at kH*kW offsets.  v_mfma_i32_16x16x64_i8 wants 16 consecutive K bytes per lane.  For G they
// are an aligned 16-byte LDS read.  For X one LDS copy per kh is staged, fetched from global memory
// at the dword below f + kh*row_pitch, so that a lane reads 24 aligned bytes (b128 + b64) per kh and
// derives the kW windows with v_alignbyte_b32 (shift (kh*row_pitch mod 4) + kw).
//
// Workgroup = 4 waves.  A wave owns a 64 (co) x 16*NB (ci) x kH*kW accumulator tile (144 VGPRs for
// 3x3, NB = 1).  The four waves either take four ci blocks (WGK = 1) or share one ci block and split
// the K steps of every staged chunk (WGK = 4, reduced through LDS at the end); the latter keeps all
// 256 CUs busy on layers with few channels.  K may also be split across workgroups: each writes its
// partial tile with coalesced stores and a second kernel sums the partials (exact, order independent)
// and de-quantizes.  Global loads run PF chunks ahead of the MFMAs through a register FIFO.
#include <algorithm>
#include <type_traits>

#include "daq_internal.h"

namespace daq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i_a4 __attribute__((ext_vector_type(4), aligned(4)));
typedef int v2i_a4 __attribute__((ext_vector_type(2), aligned(4)));
typedef int v4i_a1 __attribute__((ext_vector_type(4), aligned(1)));

constexpr int kKC = 256;          // K bytes staged per chunk (4 MFMA K-steps of 64)
constexpr int kPA = kKC + 16;     // LDS row pitch: +16 B holds the realignment slack and rotates banks between rows
constexpr int kBM = 64;           // co rows per workgroup

struct DwArgs {
    const int8_t* g;      // vq, [Cout][klen]
    const int8_t* x;      // q(X'), [Cin][chan_pitch_x]
    int64_t klen;         // bytes of the flat axis (multiple of 256)
    int64_t x_chan_pitch;
    int Cout, Cin;
    int row_pitch;        // bytes per image row of both operands
    int nchunks;          // klen / kKC
    int splits;           // workgroups along K
    int tiles_n, tiles_m; // ci tiles, co tiles
    int32_t* part;        // splits > 1: partial tiles [tile][split][wave-of-ci][reg][lane]
    // splits == 1: the tile is complete, de-quantize and store it directly
    const float* s_x;
    const float* s_chan;
    float* dW;
    int32_t* acc_out;    int bf16;             // dW is bfloat16 storage
};

__device__ __forceinline__ int alignbyte(int hi, int lo, int sh) {
    return (int)__builtin_amdgcn_alignbyte((unsigned)hi, (unsigned)lo, (unsigned)sh);
}

template <int KH, int KW, int WQ4, int WGK, int NB, int PF>
__global__ __launch_bounds__(256) void k_dw_mfma(DwArgs p) {
    constexpr int WGN = 4 / WGK;          // waves along ci
    constexpr int BN = 16 * NB * WGN;     // ci rows per workgroup
    constexpr int T = KH * KW;
    constexpr int NT = NB * T;            // accumulator tiles per co block
    constexpr int UR = kPA / 16;          // 16-byte units per staged row (17)
    constexpr int A_UNITS = kBM * (kKC / 16);
    constexpr int B_UNITS = KH * BN * UR;
    constexpr int A_PER_T = A_UNITS / 256;
    constexpr int B_PER_T = (B_UNITS + 255) / 256;
    constexpr int A_BYTES = kBM * kPA;
    constexpr int STAGE = A_BYTES + KH * BN * kPA;
    extern __shared__ __align__(16) int8_t lds[];

    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int wn = wave % WGN, wk = wave / WGN;
    const int li = lane & 15, lg = lane >> 4;

    // Workgroup i runs on XCD i % 8.  All output tiles of one K split are placed on one XCD, so a slice
    // of the two operands is fetched from HBM into a single L2 and shared there by the tiles.
    int split, tile;
    {
        const int b = blockIdx.x, tiles = p.tiles_n * p.tiles_m;
        const int full = (p.splits / kXcd) * kXcd;       // splits that fill whole rounds of 8
        const int x = b % kXcd, q = b / kXcd;
        if (q < (full / kXcd) * tiles) {
            split = (q / tiles) * kXcd + x;
            tile = q % tiles;
        } else {                                           // remainder: plain order
            const int rb = b - full * tiles;
            split = full + rb % (p.splits - full);
            tile = rb / (p.splits - full);
        }
    }
    const int tn = tile % p.tiles_n;
    const int tm = tile / p.tiles_n;
    const int co0 = tm * kBM, ci0 = tn * BN;
    const int per = p.nchunks / p.splits, rem = p.nchunks % p.splits;
    const int c_begin = split * per + min(split, rem);
    const int c_end = c_begin + per + (split < rem ? 1 : 0);

    v4i acc[4][NT];
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[m][t] = v4i{0, 0, 0, 0};

    // ---- staging: global -> register FIFO -> LDS ----
    uint4 ra[PF][A_PER_T];
    uint4 rb[PF][B_PER_T];
    // per-thread source offsets of the units this thread stages (relative to the chunk start)
    int64_t a_off[A_PER_T], b_off[B_PER_T];
    int a_lds[A_PER_T], b_lds[B_PER_T];
#pragma unroll
    for (int i = 0; i < A_PER_T; ++i) {
        const int u = tid + 256 * i;
        const int row = u / (kKC / 16), c16 = u % (kKC / 16);
        a_off[i] = (co0 + row < p.Cout) ? (int64_t)(co0 + row) * p.klen + 16 * c16 : -1;
        a_lds[i] = row * kPA + 16 * c16;
    }
#pragma unroll
    for (int i = 0; i < B_PER_T; ++i) {
        const int u = tid + 256 * i;
        const int c16 = u % UR;
        const int row = (u / UR) % BN;
        const int kh = u / (UR * BN);
        const int r0 = (kh * p.row_pitch) & 3;
        b_off[i] = (u < B_UNITS && ci0 + row < p.Cin)
                       ? (int64_t)(ci0 + row) * p.x_chan_pitch + kh * p.row_pitch - r0 + 16 * c16 : -1;
        b_lds[i] = (u < B_UNITS) ? A_BYTES + (kh * BN + row) * kPA + 16 * c16 : -1;
    }
    auto load_chunk = [&](int chunk, int set) {
        const int64_t k0 = (int64_t)chunk * kKC;
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i)
            ra[set][i] = ld16_or_zero(p.g + a_off[i] + k0, a_off[i] >= 0);
#pragma unroll
        for (int i = 0; i < B_PER_T; ++i) {
            const bool ok = b_off[i] >= 0;
            const v4i_a4 v = *reinterpret_cast<const v4i_a4*>(ok ? (const void*)(p.x + b_off[i] + k0)
                                                                 : (const void*)g_zero64);  // dword aligned only
            rb[set][i] = make_uint4((unsigned)v[0], (unsigned)v[1], (unsigned)v[2], (unsigned)v[3]);
        }
    };
    auto store_chunk = [&](int buf, int set) {
        int8_t* base = lds + buf * STAGE;
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i) *reinterpret_cast<uint4*>(base + a_lds[i]) = ra[set][i];
#pragma unroll
        for (int i = 0; i < B_PER_T; ++i)
            if (b_lds[i] >= 0) *reinterpret_cast<uint4*>(base + b_lds[i]) = rb[set][i];
    };

    if (c_begin < c_end) {
        load_chunk(c_begin, 0);
        store_chunk(0, 0);
#pragma unroll
        for (int i = 1; i <= PF; ++i)
            if (c_begin + i < c_end) load_chunk(c_begin + i, i % PF);
    }
    __syncthreads();

    for (int base = c_begin; base < c_end; base += PF) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int chunk = base + u;
            if (chunk < c_end) {
                const int buf = (chunk - c_begin) & 1;
                const int8_t* A = lds + buf * STAGE;
                const int8_t* B = A + A_BYTES;
#pragma unroll
                for (int ks = wk; ks < kKC / 64; ks += WGK) {
                    v4i a[4];
#pragma unroll
                    for (int m = 0; m < 4; ++m)
                        a[m] = *reinterpret_cast<const v4i*>(A + (16 * m + li) * kPA + ks * 64 + 16 * lg);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                        for (int kh = 0; kh < KH; ++kh) {
                            const int8_t* src = B + (kh * BN + (wn * NB + nb) * 16 + li) * kPA + ks * 64 + 16 * lg;
                            const v4i lo = *reinterpret_cast<const v4i*>(src);
                            int d[6] = {lo[0], lo[1], lo[2], lo[3], 0, 0};
                            if (KW > 1 || ((kh * WQ4) & 3) != 0) {
                                const v2i hi = *reinterpret_cast<const v2i*>(src + 16);
                                d[4] = hi[0];
                                d[5] = hi[1];
                            }
#pragma unroll
                            for (int kw = 0; kw < KW; ++kw) {
                                const int s = ((kh * WQ4) & 3) + kw;  // byte shift of this tap's window
                                const int j = s >> 2, sh = s & 3;
                                v4i bf;
                                if (sh == 0)
                                    bf = v4i{d[j], d[j + 1], d[j + 2], d[j + 3]};
                                else
                                    bf = v4i{alignbyte(d[j + 1], d[j], sh), alignbyte(d[j + 2], d[j + 1], sh),
                                             alignbyte(d[j + 3], d[j + 2], sh), alignbyte(d[j + 4], d[j + 3], sh)};
                                const int t = nb * T + kh * KW + kw;
#pragma unroll
                                for (int m = 0; m < 4; ++m)
                                    acc[m][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[m], bf, acc[m][t], 0, 0, 0);
                            }
                        }
                }
                // chunk+1 goes to the other LDS buffer; its register set is then refilled PF chunks ahead
                const int nset = (u + 1) % PF;  // a constant once the loop is unrolled
                if (chunk + 1 < c_end) store_chunk(buf ^ 1, nset);
                if (chunk + 1 + PF < c_end) load_chunk(chunk + 1 + PF, nset);
                __syncthreads();
            }
        }
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
                    for (int t = 0; t < NT; ++t)
#pragma unroll
                        for (int r = 0; r < 4; ++r) red[((m * NT + t) * 4 + r) * kWave + lane] = acc[m][t][r];
            }
            __syncthreads();
            if (wk == 0) {
#pragma unroll
                for (int m = 0; m < 4; ++m)
#pragma unroll
                    for (int t = 0; t < NT; ++t)
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[m][t][r] += red[((m * NT + t) * 4 + r) * kWave + lane];
            }
        }
        if (wk != 0) return;
    }

    if (p.splits > 1) {
        // partial tile: register q of lane l at [((tile*splits + split)*WGN + wn)*16*NT + q][l]
        int32_t* dst = p.part + (((int64_t)(tm * p.tiles_n + tn) * p.splits + split) * WGN + wn) * (16 * NT) * kWave + lane;
#pragma unroll
        for (int m = 0; m < 4; ++m)
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) dst[((m * NT + t) * 4 + r) * kWave] = acc[m][t][r];
        return;
    }

    // complete tile: de-quantize and store
    const float sx = *p.s_x / 127.0f;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int ci = ci0 + (wn * NB + nb) * 16 + li;
        if (ci >= p.Cin) continue;
#pragma unroll
        for (int m = 0; m < 4; ++m)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int co = co0 + 16 * m + 4 * lg + r;
                if (co < p.Cout) {
                    const int64_t off = ((int64_t)co * p.Cin + ci) * T;
                    const float sc = sx * (p.s_chan[co] / 127.0f);
#pragma unroll
                    for (int t = 0; t < T; ++t) {
                        store_result(p.dW, off + t, (float)acc[m][nb * T + t][r] * sc, p.bf16);
                        if (p.acc_out) p.acc_out[off + t] = acc[m][nb * T + t][r];
                    }
                }
            }
    }
}

// ---------------------------------------------------------------------------------------------
// Split-K variant for layers with few channels (one output tile per 64 x 16*NB block, many K slices).
// The four waves of a workgroup work on four disjoint runs of K steps with no barrier between them:
// a lane's MFMA fragments are 16 contiguous bytes of one channel row, so they are fetched straight
// from global memory into registers (G aligned, X at the dword below its shifted window), PFD steps
// ahead.  At the end wave m keeps co block m: the other waves hand it their part through LDS.
// ---------------------------------------------------------------------------------------------
template <int KH, int KW, int WQ4, int NB, int PFD>
__global__ __launch_bounds__(256) void k_dw_direct(DwArgs p) {
    constexpr int T = KH * KW;
    constexpr int NT = NB * T;
    extern __shared__ __align__(16) int8_t lds[];
    int* red = reinterpret_cast<int*>(lds);  // [owner 4][source 3][NT*4][64]

    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int li = lane & 15, lg = lane >> 4;
    int split, tile;
    {
        const int b = blockIdx.x, tiles = p.tiles_n * p.tiles_m;
        const int full = (p.splits / kXcd) * kXcd;
        const int x = b % kXcd, q = b / kXcd;
        if (q < (full / kXcd) * tiles) {
            split = (q / tiles) * kXcd + x;
            tile = q % tiles;
        } else {
            const int rb = b - full * tiles;
            split = full + rb % (p.splits - full);
            tile = rb / (p.splits - full);
        }
    }
    const int tn = tile % p.tiles_n, tm = tile / p.tiles_n;
    const int co0 = tm * kBM, ci0 = tn * 16 * NB;
    // K steps (64 bytes each) of this wave
    const int nsteps = p.nchunks * (kKC / 64);
    const int units = p.splits * 4, unit = split * 4 + wave;
    const int per = nsteps / units, rem = nsteps % units;
    const int s_begin = unit * per + min(unit, rem);
    const int s_end = s_begin + per + (unit < rem ? 1 : 0);

    const int8_t* ga[4];
    int gmask[4];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const int co = co0 + 16 * m + li;
        ga[m] = p.g + (int64_t)(co < p.Cout ? co : 0) * p.klen + 16 * lg;  // rows past Cout read row 0, masked to zero
        gmask[m] = (co < p.Cout) ? -1 : 0;
    }
    const int8_t* xb[NB][KH];
    int xmask[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int kh = 0; kh < KH; ++kh) {
            const int ci = ci0 + 16 * nb + li;
            const int r0 = (kh * p.row_pitch) & 3;
            xb[nb][kh] = p.x + (int64_t)(ci < p.Cin ? ci : 0) * p.x_chan_pitch + 16 * lg + kh * p.row_pitch - r0;
            xmask[nb] = (ci < p.Cin) ? -1 : 0;
        }

    v4i acc[4][NT];
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[m][t] = v4i{0, 0, 0, 0};

    v4i ra[PFD][4];
    v4i rlo[PFD][NB][KH];
    v2i rhi[PFD][NB][KH];
    auto load_step = [&](int s, int slot) {
        const int64_t k = (int64_t)s * 64;
#pragma unroll
        for (int m = 0; m < 4; ++m)
            ra[slot][m] = *reinterpret_cast<const v4i*>(gmask[m] ? (const void*)(ga[m] + k) : (const void*)g_zero64);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int kh = 0; kh < KH; ++kh) {
                const int8_t* src = xmask[nb] ? xb[nb][kh] + k : reinterpret_cast<const int8_t*>(g_zero64);
                const v4i_a4 lo = *reinterpret_cast<const v4i_a4*>(src);
                rlo[slot][nb][kh] = v4i{lo[0], lo[1], lo[2], lo[3]};
                if (KW > 1 || ((kh * WQ4) & 3) != 0) {
                    const v2i_a4 hi = *reinterpret_cast<const v2i_a4*>(src + 16);
                    rhi[slot][nb][kh] = v2i{hi[0], hi[1]};
                } else {
                    rhi[slot][nb][kh] = v2i{0, 0};
                }
            }
    };

#pragma unroll
    for (int i = 0; i < PFD; ++i)
        if (s_begin + i < s_end) load_step(s_begin + i, i);

    for (int base = s_begin; base < s_end; base += PFD) {
#pragma unroll
        for (int u = 0; u < PFD; ++u) {
            const int s = base + u;
            if (s < s_end) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int kh = 0; kh < KH; ++kh) {
                        const v4i lo = rlo[u][nb][kh];
                        const v2i hi = rhi[u][nb][kh];
                        const int d[6] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1]};
#pragma unroll
                        for (int kw = 0; kw < KW; ++kw) {
                            const int sft = ((kh * WQ4) & 3) + kw;
                            const int j = sft >> 2, sh = sft & 3;
                            v4i bf;
                            if (sh == 0)
                                bf = v4i{d[j], d[j + 1], d[j + 2], d[j + 3]};
                            else
                                bf = v4i{alignbyte(d[j + 1], d[j], sh), alignbyte(d[j + 2], d[j + 1], sh),
                                         alignbyte(d[j + 3], d[j + 2], sh), alignbyte(d[j + 4], d[j + 3], sh)};
                            const int t = nb * T + kh * KW + kw;
#pragma unroll
                            for (int m = 0; m < 4; ++m)
                                acc[m][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ra[u][m], bf, acc[m][t], 0, 0, 0);
                        }
                    }
                if (s + PFD < s_end) load_step(s + PFD, u);
            }
        }
    }

    // ---- wave m collects co block m from the other three waves ----
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        if (wave != m) {
            const int srcw = wave < m ? wave : wave - 1;
            int* dst = red + ((m * 3 + srcw) * NT * 4) * kWave + lane;
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) dst[(t * 4 + r) * kWave] = acc[m][t][r];
        }
    }
    __syncthreads();
    const float sx = *p.s_x / 127.0f;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        if (wave == m) {
#pragma unroll
            for (int w = 0; w < 3; ++w) {
                const int* src = red + ((m * 3 + w) * NT * 4) * kWave + lane;
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[m][t][r] += src[(t * 4 + r) * kWave];
            }
            if (p.splits > 1) {
                // partial tile, same slot order as the reduction kernel expects: q = (m*NT + t)*4 + r
                int32_t* dst = p.part + ((int64_t)tile * p.splits + split) * (16 * NT) * kWave + lane;
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int r = 0; r < 4; ++r) dst[((m * NT + t) * 4 + r) * kWave] = acc[m][t][r];
            } else {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const int ci = ci0 + 16 * nb + li;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int co = co0 + 16 * m + 4 * lg + r;
                        if (ci < p.Cin && co < p.Cout) {
                            const int64_t off = ((int64_t)co * p.Cin + ci) * T;
                            const float sc = sx * (p.s_chan[co] / 127.0f);
#pragma unroll
                            for (int t = 0; t < T; ++t) {
                                store_result(p.dW, off + t, (float)acc[m][nb * T + t][r] * sc, p.bf16);
                                if (p.acc_out) p.acc_out[off + t] = acc[m][nb * T + t][r];
                            }
                        }
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// General form: any filter extent, stride and dilation.  A tap (kh, kw) pairs gradient position f
// with byte  tap_off[t] + f  of an activation channel, where tap_off selects the stride-phase plane
// the tap reads and its shift inside it; the host tabulates it, the kernel never looks at the
// geometry.  Same barrier-free scheme as above: MFMA fragments straight from global memory (G
// aligned, X with byte alignment), PFD steps ahead.  Either the four waves split the K steps and
// every wave holds all taps (WTAPS = false, filters up to 3 x 3), or every wave runs all K steps
// of the workgroup on its own share of the taps (WTAPS = true; 4 or 8 waves, up to 56 taps, e.g. 7 x 7).
// Rows past Cout / Cin and unused tap slots compute on valid memory and are never stored.
// ---------------------------------------------------------------------------------------------
constexpr int kMaxTapSlots = 56;
struct TapTable {
    int64_t off[kMaxTapSlots];   // byte offset of the tap's window start inside an activation channel
    int id[kMaxTapSlots];        // kh*kW + kw, or -1 for an unused slot
    int T;                       // kH * kW
    // Row mode, for layers with very few input channels (an RGB stem): the rows of the activation operand are the
    // (ci, kw) pairs, row ci*kW + kw reading channel ci at row_off[kw], and the "taps" are the kh alone (T = kH,
    // id = kh).  3 x 7 rows fill 21 of 32 lanes where channel rows would fill 3 of 16, and a tap slot covers a whole
    // filter row.  0 = off.
    int row_kw;
    int64_t row_off[8];
};

template <int TW, int NB, int PFD, bool WTAPS, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void k_dw_taps(DwArgs p, TapTable tt) {
    static_assert(WTAPS || WAVES == 4, "the K-splitting form hands tiles over between exactly four waves");
    static_assert(WAVES * TW <= kMaxTapSlots, "tap table too small");
    constexpr int NT = NB * TW;
    extern __shared__ __align__(16) int8_t lds[];
    int* red = reinterpret_cast<int*>(lds);  // !WTAPS: [owner 4][source 3][NT*4][64]

    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int li = lane & 15, lg = lane >> 4;
    int split, tile;
    {
        const int b = blockIdx.x, tiles = p.tiles_n * p.tiles_m;
        const int full = (p.splits / kXcd) * kXcd;
        const int x = b % kXcd, q = b / kXcd;
        if (q < (full / kXcd) * tiles) {
            split = (q / tiles) * kXcd + x;
            tile = q % tiles;
        } else {
            const int rb = b - full * tiles;
            split = full + rb % (p.splits - full);
            tile = rb / (p.splits - full);
        }
    }
    const int tn = tile % p.tiles_n, tm = tile / p.tiles_n;
    const int co0 = tm * kBM, ci0 = tn * 16 * NB;
    // K steps (64 bytes each) of this wave
    const int nsteps = p.nchunks * (kKC / 64);
    const int units = WTAPS ? p.splits : p.splits * 4;
    const int unit = WTAPS ? split : split * 4 + wave;
    const int per = nsteps / units, rem = nsteps % units;
    const int s_begin = unit * per + min(unit, rem);
    const int s_end = s_begin + per + (unit < rem ? 1 : 0);

    // Addresses are a wave-uniform 64-bit base (operand + tap offset + K position, kept in scalar registers)
    // plus a 32-bit per-lane offset (row and 16-byte K group); both operands are smaller than 2 GiB.
    uint32_t va[4], vb[NB];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const int co = co0 + 16 * m + li;
        va[m] = (uint32_t)((int64_t)(co < p.Cout ? co : 0) * p.klen + 16 * lg);
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        if (tt.row_kw) {   // uniform
            const int R = 16 * nb + li, ci = R / tt.row_kw, kw = R - ci * tt.row_kw;
            int64_t ro = tt.row_off[0];
#pragma unroll
            for (int q = 1; q < 8; ++q) ro = (kw == q) ? tt.row_off[q] : ro;
            vb[nb] = (uint32_t)((int64_t)(ci < p.Cin ? ci : 0) * p.x_chan_pitch + (ci < p.Cin ? ro : 0) + 16 * lg);
        } else {
            const int ci = ci0 + 16 * nb + li;
            vb[nb] = (uint32_t)((int64_t)(ci < p.Cin ? ci : 0) * p.x_chan_pitch + 16 * lg);
        }
    }
    // wave-uniform tap offsets and ids; the table is indexed with constants only (a run-time index into a
    // by-value kernel argument would make the compiler copy it to scratch memory)
    int64_t toff[TW];
    int tid_of[TW];
#pragma unroll
    for (int j = 0; j < TW; ++j) {
        toff[j] = tt.off[j];
        tid_of[j] = tt.id[j];
        if (WTAPS) {
#pragma unroll
            for (int w = 1; w < WAVES; ++w)
                if (wave == w) { toff[j] = tt.off[w * TW + j]; tid_of[j] = tt.id[w * TW + j]; }
        }
    }

    v4i acc[4][NT];
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[m][t] = v4i{0, 0, 0, 0};

    v4i ra[PFD][4];
    v4i rb[PFD][NT];
    auto load_step = [&](int s, int slot) {
        const int64_t k = (int64_t)s * 64;
        const int8_t* gk = p.g + k;
#pragma unroll
        for (int m = 0; m < 4; ++m) ra[slot][m] = *reinterpret_cast<const v4i*>(gk + va[m]);
#pragma unroll
        for (int j = 0; j < TW; ++j) {
            const int8_t* xk = p.x + (toff[j] + k);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const v4i_a1 v = *reinterpret_cast<const v4i_a1*>(xk + vb[nb]);
                rb[slot][nb * TW + j] = v4i{v[0], v[1], v[2], v[3]};
            }
        }
    };

#pragma unroll
    for (int i = 0; i < PFD; ++i)
        if (s_begin + i < s_end) load_step(s_begin + i, i);

    for (int base = s_begin; base < s_end; base += PFD) {
#pragma unroll
        for (int u = 0; u < PFD; ++u) {
            const int s = base + u;
            if (s < s_end) {
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int m = 0; m < 4; ++m)
                        acc[m][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ra[u][m], rb[u][t], acc[m][t], 0, 0, 0);
                if (s + PFD < s_end) load_step(s + PFD, u);
            }
        }
    }

    const float sx = *p.s_x / 127.0f;
    const int T = tt.T;
    // stores accumulator (m, nb, j) of this wave; partial layout q = (m*(NB*T) + nb*T + tap)*4 + r
    auto emit = [&](auto mc) __attribute__((always_inline)) {
        constexpr int m = decltype(mc)::value;
        int32_t* part = p.part + ((int64_t)tile * p.splits + split) * (16 * NB * T) * kWave + lane;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int ci = ci0 + 16 * nb + li;
#pragma unroll
            for (int j = 0; j < TW; ++j) {
                const int tap = tid_of[j];
                if (tap < 0) continue;   // wave-uniform
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int v = acc[m][nb * TW + j][r];
                    if (p.splits > 1) {
                        part[(int64_t)((m * NB * T + nb * T + tap) * 4 + r) * kWave] = v;
                    } else {
                        const int co = co0 + 16 * m + 4 * lg + r;
                        int cin = ci;
                        int64_t off = ((int64_t)co * p.Cin + ci) * T + tap;
                        if (tt.row_kw) {   // row (ci, kw), tap kh
                            const int R = 16 * nb + li;
                            cin = R / tt.row_kw;
                            off = (((int64_t)co * p.Cin + cin) * T + tap) * tt.row_kw + (R - cin * tt.row_kw);
                        }
                        if (cin < p.Cin && co < p.Cout) {
                            store_result(p.dW, off, (float)v * (sx * (p.s_chan[co] / 127.0f)), p.bf16);
                            if (p.acc_out) p.acc_out[off] = v;
                        }
                    }
                }
            }
        }
    };

    if (WTAPS) {
        emit(std::integral_constant<int, 0>{});
        emit(std::integral_constant<int, 1>{});
        emit(std::integral_constant<int, 2>{});
        emit(std::integral_constant<int, 3>{});
        return;
    }
    // ---- wave m collects co block m from the other three waves ----
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        if (wave != m) {
            const int srcw = wave < m ? wave : wave - 1;
            v4i* dst = reinterpret_cast<v4i*>(red) + ((m * 3 + srcw) * NT) * kWave + lane;   // [tile][lane]: 16-byte accesses
#pragma unroll
            for (int t = 0; t < NT; ++t) dst[t * kWave] = acc[m][t];
        }
    }
    __syncthreads();
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        if (wave == m) {
#pragma unroll
            for (int w = 0; w < 3; ++w) {
                const v4i* src = reinterpret_cast<const v4i*>(red) + ((m * 3 + w) * NT) * kWave + lane;
#pragma unroll
                for (int t = 0; t < NT; ++t) acc[m][t] += src[t * kWave];
            }
        }
    }
    if (wave == 0) emit(std::integral_constant<int, 0>{});
    if (wave == 1) emit(std::integral_constant<int, 1>{});
    if (wave == 2) emit(std::integral_constant<int, 2>{});
    if (wave == 3) emit(std::integral_constant<int, 3>{});
}

// Sum of the K-split partial tiles, then dW[co][...] = acc * ((s_x/127) * (s_chan[co]/127)).
// A workgroup owns 64 consecutive slots of the partial layout (one 256-byte run per split); its four
// waves take every fourth split with eight loads in flight each and combine through LDS.
__global__ __launch_bounds__(256) void k_dw_reduce(const int32_t* __restrict__ part, int64_t runs, int splits, int tiles_n, int wgn,
                                                   int nb_per_wave, int T, int row_kw, int Cout, int Cin, const float* s_x,
                                                   const float* __restrict__ s_chan, float* __restrict__ dW,
                                                   int32_t* __restrict__ acc_out, int bf16) {
    const int lane = threadIdx.x % kWave, grp = threadIdx.x / kWave;
    const int NT = nb_per_wave * T;
    const int per_wave = 16 * NT * kWave;
    // with few splits every wave sums a run of 64 slots alone (all loads in flight, no LDS); else the four waves share one
    const bool alone = splits <= 16;
    const int64_t run = alone ? (int64_t)blockIdx.x * 4 + grp : (int64_t)blockIdx.x;
    if (run >= runs) return;   // uniform per wave; only in the `alone` mode, which has no barrier
    const int64_t i = run * kWave + lane;   // slot
    const int q = (int)((i / kWave) % (16 * NT));
    const int wn = (int)((i / per_wave) % wgn);
    const int tile = (int)(i / ((int64_t)per_wave * wgn));
    const int64_t stride = (int64_t)per_wave * wgn;          // between consecutive splits of a tile
    const int32_t* src = part + (int64_t)tile * splits * stride + (int64_t)wn * per_wave + (int64_t)q * kWave + lane;
    int32_t a = 0;
    if (alone) {
        int32_t v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = src[(int64_t)min(u, splits - 1) * stride];
#pragma unroll
        for (int u = 0; u < 16; ++u) a += u < splits ? v[u] : 0;
    } else {
        int s = grp;
        for (; s + 28 < splits; s += 32) {
            int32_t v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = src[(int64_t)(s + 4 * u) * stride];
#pragma unroll
            for (int u = 0; u < 8; ++u) a += v[u];
        }
        for (; s < splits; s += 4) a += src[(int64_t)s * stride];
        __shared__ int32_t l_sum[4][kWave];
        l_sum[grp][lane] = a;
        __syncthreads();
        if (grp != 0) return;
        a = l_sum[0][lane] + l_sum[1][lane] + l_sum[2][lane] + l_sum[3][lane];
    }
    const int r = q & 3, t_all = (q >> 2) % NT, m = (q >> 2) / NT;
    const int nb = t_all / T, t = t_all % T;
    const int tm = tile / tiles_n, tn = tile % tiles_n;
    const int co = tm * kBM + 16 * m + 4 * (lane >> 4) + r;
    int ci = tn * (16 * nb_per_wave * wgn) + (wn * nb_per_wave + nb) * 16 + (lane & 15);
    int64_t off = ((int64_t)co * Cin + ci) * T + t;
    if (row_kw) {   // row mode of the tap-table kernel: the row is (ci, kw), the tap is kh
        const int R = nb * 16 + (lane & 15);
        ci = R / row_kw;
        off = (((int64_t)co * Cin + ci) * T + t) * row_kw + (R - ci * row_kw);
    }
    if (co >= Cout || ci >= Cin) return;
    store_result(dW, off, (float)a * ((*s_x / 127.0f) * (s_chan[co] / 127.0f)), bf16);
    if (acc_out) acc_out[off] = a;
}

struct Plan {
    bool ok;
    bool general;         // tap-table kernel (any extent, stride, dilation)
    int tw;               // general: tap slots per wave
    bool wtaps;           // general: waves split the taps instead of K
    int row_kw;           // general: kW when the activation rows are (ci, kw) pairs (few input channels), else 0
    int kh, wgk, nb, pf, splits, tiles_m, tiles_n, nchunks;
    size_t lds_bytes;
    int64_t part_slots;   // int32 slots of one split's worth of partial tiles
};

// Plan of the tap-table kernel.
Plan make_general_plan(const daq_conv_desc& d) {
    Plan pl{};
    const int T = d.kH * d.kW;
    if (d.groups != 1 || T > kMaxTapSlots) return pl;
    daq_layout Lg;
    if (daq_layout_vq(&d, &Lg) != DAQ_OK) return pl;
    pl.general = true;
    pl.kh = d.kH;
    pl.nchunks = (int)(Lg.plane_pitch / kKC);
    const bool rowmode = T > 9 && d.Cin * d.kW <= 32 && d.kH <= 8 && d.kW <= 8;
    if (rowmode) { pl.row_kw = d.kW; pl.tw = 2; pl.nb = 2; pl.wtaps = true; pl.pf = 3; }   // taps = kh, two per wave
    else if (T == 1) { pl.tw = 1; pl.nb = 4; pl.wtaps = false; pl.pf = 4; }
    else if (T <= 9) { pl.tw = 9; pl.nb = 1; pl.wtaps = false; pl.pf = 3; }
    else { pl.tw = 7; pl.nb = 1; pl.wtaps = true; pl.pf = 2; }   // 4 waves up to 28 taps, 8 waves beyond
    pl.wgk = pl.wtaps ? 1 : 4;
    pl.tiles_m = (int)ceil_div(d.Cout, kBM);
    pl.tiles_n = pl.row_kw ? 1 : (int)ceil_div(d.Cin, 16 * pl.nb);
    const int64_t tiles = (int64_t)pl.tiles_m * pl.tiles_n;
    const int64_t nsteps = (int64_t)pl.nchunks * (kKC / 64);
    int64_t s = ceil_div(512, tiles);
    const int64_t max_by_steps = std::max<int64_t>(1, nsteps / (pl.wtaps ? 2 : 8));   // at least two steps per wave
    if (s > max_by_steps) s = max_by_steps;
    // partial tiles are written and read once: keep that below ~2x the operand bytes
    const int64_t operand = (int64_t)d.Cout * Lg.plane_pitch + (int64_t)d.Cin * Lg.plane_pitch * d.strideH * d.strideW;
    const int64_t Tp = pl.row_kw ? d.kH : T;   // tap slots of the partial layout
    const int64_t tile_bytes = tiles * kBM * 16 * pl.nb * Tp * 4;
    const int64_t max_by_traffic = std::max<int64_t>(1, operand / tile_bytes);
    if (s > max_by_traffic) s = max_by_traffic;
    pl.splits = (int)std::max<int64_t>(1, s);
    pl.lds_bytes = pl.wtaps ? 256 : (size_t)12 * pl.nb * pl.tw * 4 * kWave * 4;
    if (pl.lds_bytes > 160 * 1024) return pl;
    pl.part_slots = tiles * 16 * pl.nb * Tp * kWave;
    pl.ok = true;
    return pl;
}

Plan make_plan(const daq_conv_desc& d) {
    Plan pl{};
    pl.ok = false;
    if (d.groups != 1) return pl;
    const bool unit = d.strideH == 1 && d.strideW == 1 && d.dilH == 1 && d.dilW == 1;
    const bool tuned = unit && d.kH == 3 && d.kW == 3;
    if (!tuned) return make_general_plan(d);
    daq_layout Lg;
    if (daq_layout_vq(&d, &Lg) != DAQ_OK) return pl;
    pl.kh = d.kH;
    pl.nchunks = (int)(Lg.plane_pitch / kKC);
    pl.tiles_m = (int)ceil_div(d.Cout, kBM);
    const int T = d.kH * d.kW;
    pl.nb = 1;
    const int ci_wave = 16 * pl.nb;
    // Prefer a shape with enough output tiles to fill the 256 CUs without splitting K (one launch).
    // With few channels the four waves of a workgroup split K instead of ci, and K is also split
    // across workgroups, bounded by the partial-tile traffic it causes.
    const int64_t tiles1 = (int64_t)pl.tiles_m * ceil_div(d.Cin, 4 * ci_wave);
    const int64_t tiles4 = (int64_t)pl.tiles_m * ceil_div(d.Cin, ci_wave);
    int64_t s = 1;
    if (tiles1 >= 192) {
        pl.wgk = 1;
    } else {
        pl.wgk = 4;
        if (tiles4 < 192) {
            s = ceil_div(256, tiles4);
            const int64_t max_by_chunks = pl.nchunks / 2 > 0 ? pl.nchunks / 2 : 1;
            if (s > max_by_chunks) s = max_by_chunks;
            // partial tiles are written and read once: keep that below ~2x the operand bytes
            const int64_t operand = (int64_t)(d.Cout + d.Cin) * Lg.plane_pitch;
            const int64_t tile_bytes = (int64_t)pl.tiles_m * kBM * ceil_div(d.Cin, ci_wave) * ci_wave * T * 4;
            const int64_t max_by_traffic = operand / tile_bytes > 0 ? operand / tile_bytes : 1;
            if (s > max_by_traffic) s = max_by_traffic;
            if (s < 1) s = 1;
        }
    }
    pl.pf = (pl.wgk == 4) ? 4 : 1;
    const int wgn = 4 / pl.wgk;
    const int bn = ci_wave * wgn;
    pl.tiles_n = (int)ceil_div(d.Cin, bn);
    pl.splits = (int)s;
    const size_t stage = (size_t)kBM * kPA + (size_t)d.kH * bn * kPA;
    pl.lds_bytes = 2 * stage;
    if (pl.wgk > 1) pl.lds_bytes = (size_t)12 * pl.nb * T * 4 * kWave * 4;  // direct kernel: hand-over area only
    if (pl.lds_bytes > 160 * 1024) return pl;
    pl.part_slots = (int64_t)pl.tiles_m * pl.tiles_n * wgn * 16 * pl.nb * T * kWave;
    pl.ok = true;
    return pl;
}

template <int KH, int KW, int WGK, int NB, int PF>
daq_status launch_dw(const Plan& pl, const DwArgs& a, int wq4, hipStream_t st) {
    const dim3 grid((unsigned)(pl.tiles_m * pl.tiles_n * pl.splits));
#define DAQ_DW_CASE(Q)                                                                                            \
    if (wq4 == Q) {                                                                                               \
        auto kern = k_dw_mfma<KH, KW, Q, WGK, NB, PF>;                                                            \
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,                    \
                                (int)pl.lds_bytes) != hipSuccess)                                                 \
            return DAQ_ERR_HIP;                                                                                   \
        DAQ_LAUNCH("conv_bwd_filter_frag", st, hipLaunchKernelGGL(kern, grid, dim3(256), pl.lds_bytes, st, a));   \
        return DAQ_OK;                                                                                            \
    }
    DAQ_DW_CASE(0) DAQ_DW_CASE(1) DAQ_DW_CASE(2) DAQ_DW_CASE(3)
#undef DAQ_DW_CASE
    return DAQ_ERR_UNSUPPORTED;
}

template <int KH, int KW, int NB, int PFD>
daq_status launch_dw_direct(const Plan& pl, const DwArgs& a, int wq4, hipStream_t st) {
    const dim3 grid((unsigned)(pl.tiles_m * pl.tiles_n * pl.splits));
#define DAQ_DW_CASE(Q)                                                                                            \
    if (wq4 == Q) {                                                                                               \
        auto kern = k_dw_direct<KH, KW, Q, NB, PFD>;                                                              \
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,                    \
                                (int)pl.lds_bytes) != hipSuccess)                                                 \
            return DAQ_ERR_HIP;                                                                                   \
        DAQ_LAUNCH("conv_bwd_filter_direct_frag", st, hipLaunchKernelGGL(kern, grid, dim3(256), pl.lds_bytes, st, a));   \
        return DAQ_OK;                                                                                            \
    }
    DAQ_DW_CASE(0) DAQ_DW_CASE(1) DAQ_DW_CASE(2) DAQ_DW_CASE(3)
#undef DAQ_DW_CASE
    return DAQ_ERR_UNSUPPORTED;
}

template <int TW, int NB, int PFD, bool WTAPS, int WAVES>
daq_status launch_dw_taps(const Plan& pl, const DwArgs& a, const TapTable& tt, hipStream_t st) {
    const dim3 grid((unsigned)(pl.tiles_m * pl.tiles_n * pl.splits));
    auto kern = k_dw_taps<TW, NB, PFD, WTAPS, WAVES>;
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.lds_bytes) != hipSuccess)
        return DAQ_ERR_HIP;
    DAQ_LAUNCH("conv_bwd_filter_taps", st, hipLaunchKernelGGL(kern, grid, dim3(64 * WAVES), pl.lds_bytes, st, a, tt));
    return DAQ_OK;
}

// Window start of every tap inside an activation channel: the stride-phase plane it reads plus its
// shift there.  With P = padded coordinate (h + pad), tap kh reads P = ho*stride + kh*dil, i.e. phase
// (kh*dil) % stride at row ho + (kh*dil) / stride; unit stride is the one-phase case.
TapTable make_tap_table(const daq_conv_desc& d, const daq_layout& Lx, const Plan& pl) {
    TapTable tt{};
    tt.T = d.kH * d.kW;
    for (int j = 0; j < kMaxTapSlots; ++j) { tt.off[j] = 0; tt.id[j] = -1; }
    tt.row_kw = pl.row_kw;
    for (int q = 0; q < 8; ++q) tt.row_off[q] = 0;
    if (pl.row_kw) {
        // offset = [phase_h plane + row shift] (the tap, kh) + [phase_w plane + column shift] (the row's kw)
        tt.T = d.kH;
        for (int kh = 0; kh < d.kH; ++kh) {
            tt.off[kh] = (int64_t)((kh * d.dilH) % Lx.phases_h) * Lx.phases_w * Lx.plane_pitch +
                         (int64_t)(kh * d.dilH / Lx.phases_h) * Lx.row_pitch;
            tt.id[kh] = kh;
        }
        for (int kw = 0; kw < d.kW; ++kw)
            tt.row_off[kw] = (int64_t)((kw * d.dilW) % Lx.phases_w) * Lx.plane_pitch + (kw * d.dilW / Lx.phases_w);
        return tt;
    }
    for (int kh = 0; kh < d.kH; ++kh)
        for (int kw = 0; kw < d.kW; ++kw) {
            const int t = kh * d.kW + kw;
            const int ph = (kh * d.dilH) % Lx.phases_h, pw = (kw * d.dilW) % Lx.phases_w;
            tt.off[t] = (int64_t)(ph * Lx.phases_w + pw) * Lx.plane_pitch +
                        (int64_t)(kh * d.dilH / Lx.phases_h) * Lx.row_pitch + (kw * d.dilW / Lx.phases_w);
            tt.id[t] = t;
        }
    (void)pl;
    return tt;
}

}  // namespace

bool bwd_filter_mfma_supported(const daq_conv_desc& d) { return make_plan(d).ok; }

size_t bwd_filter_mfma_ws_bytes(const daq_conv_desc& d) {
    const Plan pl = make_plan(d);
    if (!pl.ok || pl.splits == 1) return 0;
    return (size_t)round_up(pl.part_slots * pl.splits * 4, 256);
}

daq_status conv_bwd_filter_mfma(const daq_conv_desc& d, const int8_t* qx, const float* s_x, const int8_t* vq,
                                const float* s_chan, float* dW, int32_t* acc, void* ws, hipStream_t st, bool bf16) {
    const Plan pl = make_plan(d);
    if (!pl.ok) return DAQ_ERR_UNSUPPORTED;
    daq_layout Lx, Lg;
    if (daq_layout_qx_cnhw(&d, &Lx) != DAQ_OK || daq_layout_vq(&d, &Lg) != DAQ_OK) return DAQ_ERR_INVALID_ARG;
    const int T = d.kH * d.kW;
    DwArgs a{};
    a.g = vq;
    a.x = qx;
    a.klen = Lg.plane_pitch;
    a.x_chan_pitch = Lx.chan_pitch;
    a.Cout = d.Cout;
    a.Cin = d.Cin;
    a.row_pitch = Lx.row_pitch;
    a.nchunks = pl.nchunks;
    a.splits = pl.splits;
    a.tiles_n = pl.tiles_n;
    a.tiles_m = pl.tiles_m;
    a.part = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(ws) + 256);
    a.s_x = s_x;
    a.s_chan = s_chan;
    a.dW = dW;
    a.acc_out = acc;
    a.bf16 = bf16 ? 1 : 0;
    daq_status rc;
    const int wq4 = Lx.row_pitch & 3;
    if (pl.general) {
        const TapTable tt = make_tap_table(d, Lx, pl);
        if (pl.row_kw) rc = launch_dw_taps<2, 2, 3, true, 4>(pl, a, tt, st);
        else if (pl.tw == 1) rc = launch_dw_taps<1, 4, 4, false, 4>(pl, a, tt, st);
        else if (pl.tw == 9) rc = launch_dw_taps<9, 1, 3, false, 4>(pl, a, tt, st);
        else if (T <= 28) rc = launch_dw_taps<7, 1, 2, true, 4>(pl, a, tt, st);
        else rc = launch_dw_taps<7, 1, 2, true, 8>(pl, a, tt, st);
    } else {
        rc = (pl.wgk == 4) ? launch_dw_direct<3, 3, 1, 3>(pl, a, wq4, st) : launch_dw<3, 3, 1, 1, 1>(pl, a, wq4, st);
    }
    if (rc != DAQ_OK) return rc;
    if (pl.splits > 1) {
        const int wgn = pl.general ? 1 : 4 / pl.wgk;
        const int64_t runs = pl.part_slots / kWave;
        const unsigned rblocks = (unsigned)(pl.splits <= 16 ? ceil_div(runs, 4) : runs);
        DAQ_LAUNCH("dw_reduce", st,
                   hipLaunchKernelGGL(k_dw_reduce, dim3(rblocks), dim3(256), 0, st,
                                      a.part, runs, pl.splits, pl.tiles_n, wgn, pl.nb, pl.row_kw ? d.kH : T, pl.row_kw, d.Cout, d.Cin,
                                      s_x, s_chan, dW, acc, bf16 ? 1 : 0));
    }
    return DAQ_OK;
}

}  // namespace daq
