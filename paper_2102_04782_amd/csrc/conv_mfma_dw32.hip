// Filter gradient  q(G_W) = q(X') (x) vq(G')  for 3 x 3 (k_dw32) and 1 x 1 (k_dw11) filters at unit stride and
// dilation, on the full-rate v_mfma_i32_32x32x32_i8 with both operands staged through LDS.
//
// Same shifted-correlation form as conv_mfma_dw.hip:
//     acc[co][ci][kh][kw] = sum_f  G[co][f] * X[ci][f + kh*row_pitch + kw]
// A workgroup stages, per 256-byte chunk of the flat axis, 32*WM gradient rows and 32*WN activation
// rows (the latter 256 + 2*row_pitch + 2 bytes long: every tap's window of the chunk) with
// coalesced loads, double buffered in LDS behind a register ring that keeps the loads of the next
// chunks in flight.  A wave owns a 32 (co) x 32 (ci) x 9 (tap) accumulator tile (144 registers).
// Its gradient fragment is one aligned 16-byte LDS read; for each filter row it reads the 24 bytes
// from the dword at or below the row's first window (activation rows have a pitch of 4 * odd bytes,
// so the 32 rows of a fragment fall into different banks, at the price of dword-aligned accesses)
// and derives the three kw windows with v_alignbyte_b32 (shift (kh*row_pitch mod 4) + kw, a
// compile-time constant per instantiation).  Waves either hold different tiles (WK = 1, four waves,
// 64 x 64 per workgroup) or share one tile and take one of the eight K steps of every chunk each
// (WK = 8: two waves per SIMD, so that one's LDS phase overlaps the other's multiplies), combined in
// parallel through LDS at the end; the latter keeps all CUs busy on layers with few channels.  K
// can also be split across workgroups: partial tiles are written with coalesced stores and summed
// by k_dw_reduce.
#include <algorithm>

#include "daq_internal.h"
#include "dw_tail.h"

namespace daq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef int v4i_a4 __attribute__((ext_vector_type(4), aligned(4)));
typedef int v2i_a4 __attribute__((ext_vector_type(2), aligned(4)));

constexpr int kKC = 256;        // K bytes staged per chunk (8 MFMA K-steps of 32)
constexpr int kPA = kKC + 16;   // LDS pitch of a gradient row: 16-byte aligned, rotates banks between rows
constexpr int kT = 9;
constexpr int kDwReducePerWave = 16;   // up to this many K splits a wave of the reduction sums a group of results alone

struct Dw32Args {
    const int8_t* g;      // vq, [Cout][klen]
    const int8_t* x;      // q(X'), [Cin][x_chan_pitch]
    int64_t klen;
    int64_t x_chan_pitch;
    int64_t x_plane_pitch;   // stride 2: bytes of one stride-phase plane of an activation channel
    int Cout, Cin;
    int row_pitch;
    int pb;               // LDS pitch of an activation row in bytes (a multiple of 4 with pb/4 odd)
    int b_units;          // 16-byte units of an activation row that are staged per chunk
    int nchunks, splits;
    int bands_m, bands_n;  // > 0: fewer than eight K splits, the tile grid is cut into bands_m x bands_n rectangles (dw_block_map)
    int band_m, band_n;    // tiles per rectangle along co and ci
    int tiles_n, tiles_m;
    int32_t* part;        // splits > 1: [tile][split][wave tile][slot = tap*16 + reg][lane]
    const float* s_x;
    const float* s_chan;
    float* dW;
    int32_t* acc_out;    int bf16;              // dW is bfloat16 storage
};

__device__ __forceinline__ int alignbyte(int hi, int lo, int sh) {
    return (int)__builtin_amdgcn_alignbyte((unsigned)hi, (unsigned)lo, (unsigned)sh);
}

// Block -> (K split, output tile).  Workgroup b runs on XCD b % 8, and what an XCD's workgroups read together is what
// its L2 has to fetch.  With eight or more splits an XCD takes whole splits: every tile of the split, i.e. one K slice
// of every operand row - each byte of the operands enters exactly one L2.  With 1, 2 or 4 splits the eight XCDs share a
// split among 8, 4 or 2 of them, and each takes a rectangle of the tile grid (bands_m x bands_n rectangles per split,
// chosen on the host to minimise rows of G plus rows of X per rectangle) instead of tiles dealt round-robin, which
// made every XCD read nearly all rows of one operand.  Returns false for the padding of the grid.
__device__ __forceinline__ bool dw_block_map(const Dw32Args& p, int& split, int& tile) {
    const int b = blockIdx.x, tiles = p.tiles_n * p.tiles_m;
    const int x = b % kXcd, q = b / kXcd;
    if (p.bands_m > 0) {
        split = x % p.splits;
        const int rect = x / p.splits;
        const int rm = rect / p.bands_n, rn = rect % p.bands_n;
        const int lm = q / p.band_n, ln = q % p.band_n;
        const int tm = rm * p.band_m + lm, tn = rn * p.band_n + ln;
        if (lm >= p.band_m || tm >= p.tiles_m || tn >= p.tiles_n) return false;
        tile = tm * p.tiles_n + tn;
        return true;
    }
    const int full = (p.splits / kXcd) * kXcd;
    if (q < (full / kXcd) * tiles) {
        split = (q / tiles) * kXcd + x;
        tile = q % tiles;
    } else {
        const int rb = b - full * tiles;
        split = full + rb % (p.splits - full);
        tile = rb / (p.splits - full);
    }
    return true;
}

// WQ4 = row_pitch mod 4.  WM x WN x WK = 4 or 8 waves: tiles along co, along ci, split of the K steps.
// PF = chunks whose global loads are in flight beyond the one being written to LDS (register ring).
//
// S2: the same product for a 3 x 3 filter at stride 2.  The activation is stored as its four stride-phase planes
// (row parity, column parity), each with the gradient's slot geometry, so tap (kh, kw) pairs gradient byte f with byte
// f + (kh/2)*row_pitch + kw/2 of plane (kh%2, kw%2): still shifted correlations over the flat axis, now against four
// staged rows per input channel (windows of 256 + row_pitch + 1 bytes).  Six 24-byte reads per K step - one per
// (plane, row shift) - serve the nine taps.
template <int WQ4, int WM, int WN, int WK, int PF, bool S2 = false>
__global__ __launch_bounds__(64 * WM * WN * WK) void k_dw32(Dw32Args p) {
    constexpr int WAVES = WM * WN * WK, NT = 64 * WAVES;
    static_assert(WAVES == 4 || WAVES == 8, "four or eight waves");
    static_assert(!S2 || (WM == 1 && WN == 1 && WK == 8), "the strided form shares one tile among eight waves");
    constexpr int BM = 32 * WM, BN = 32 * WN;
    constexpr int PL = S2 ? 4 : 1;                    // staged rows per input channel (stride-phase planes)
    constexpr int A_PER_T = BM * (kKC / 16) / NT;    // 16-byte units of the gradient tile per thread
    constexpr int A_BYTES = BM * kPA;
    constexpr int B_MAX = S2 ? 5 : 4 * WN * 256 / NT;  // 16-byte units of the activation tile per thread, at most
    extern __shared__ __align__(16) int8_t lds[];

    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int wk = wave % WK, wn = (wave / WK) % WN, wm = wave / (WK * WN);
    const int l32 = lane & 31, lh = lane >> 5;
    const int B_BYTES = PL * BN * p.pb;
    const int STAGE = A_BYTES + B_BYTES;

    int split, tile;
    if (!dw_block_map(p, split, tile)) return;   // uniform
    const int tn = tile % p.tiles_n, tm = tile / p.tiles_n;
    const int co0 = tm * BM, ci0 = tn * BN;
    const int per = p.nchunks / p.splits, rem = p.nchunks % p.splits;
    const int c_begin = split * per + min(split, rem);
    const int c_end = c_begin + per + (split < rem ? 1 : 0);

    // a complete tile is de-quantized here: its scales are requested now, long before they are needed
    float sx = 0.0f, sc_row[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (p.splits == 1) {   // uniform
        sx = *p.s_x / 127.0f;
        if constexpr (WK > 1) {
#pragma unroll
            for (int i = 0; i < 4; ++i) sc_row[i] = p.s_chan[min(co0 + wave + WAVES * i, p.Cout - 1)];   // the rows this wave stores
        }
    }

    // ---- staging assignment ----
    // gradient: unit u = tid + 256*i -> row u / 16, 16-byte column u % 16
    uint32_t a_src[A_PER_T];
    int a_dst[A_PER_T];
#pragma unroll
    for (int i = 0; i < A_PER_T; ++i) {
        const int u = tid + NT * i;
        const int row = u >> 4, c16 = u & 15;
        const int co = co0 + row;
        a_src[i] = (uint32_t)((int64_t)(co < p.Cout ? co : 0) * p.klen + 16 * c16);   // rows past Cout recompute row 0, never stored
        a_dst[i] = row * kPA + 16 * c16;
    }
    // activation: unit u = tid + 256*i of the BN x b_units tile (row-major): consecutive lanes, consecutive 16 bytes
    uint32_t b_src[B_MAX];
    int b_dst[B_MAX];
    const int b_total = PL * BN * p.b_units;
#pragma unroll
    for (int i = 0; i < B_MAX; ++i) {
        const int u = tid + NT * i;
        const int uc = u < b_total ? u : 0;
        const int row = uc / p.b_units, col = uc - row * p.b_units;   // staged row = plane * BN + channel of the tile
        const int ci = ci0 + row % BN;
        b_src[i] = (uint32_t)((int64_t)(ci < p.Cin ? ci : 0) * p.x_chan_pitch + (int64_t)(row / BN) * p.x_plane_pitch + 16 * col);
        b_dst[i] = u < b_total ? A_BYTES + row * p.pb + 16 * col : -1;
    }
    // Every call issues the same loads (past the end the last chunk is fetched again, which the caches absorb):
    // only then can the compiler count the loads in flight and wait for exactly the oldest set.
    v4i ra[PF][A_PER_T], rb[PF][B_MAX];
    const int c_last = max(c_end - 1, 0);
    auto load_chunk = [&](int chunk, int set) {
        const int64_t k0 = (int64_t)min(chunk, c_last) * kKC;
        const int8_t* gk = p.g + k0;
        const int8_t* xk = p.x + k0;
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i) ra[set][i] = *reinterpret_cast<const v4i*>(gk + a_src[i]);
#pragma unroll
        for (int i = 0; i < B_MAX; ++i) rb[set][i] = *reinterpret_cast<const v4i*>(xk + b_src[i]);
        __builtin_amdgcn_sched_barrier(0);   // keep the sets in program order
    };
    auto store_chunk = [&](int buf, int set) {
        int8_t* base = lds + buf * STAGE;
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i) *reinterpret_cast<v4i*>(base + a_dst[i]) = ra[set][i];
#pragma unroll
        for (int i = 0; i < B_MAX; ++i)
            if (b_dst[i] >= 0) *reinterpret_cast<v4i_a4*>(base + b_dst[i]) = rb[set][i];   // rows are only dword aligned
    };

    v16i acc[kT];
#pragma unroll
    for (int t = 0; t < kT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0;

    // chunk c_begin goes to LDS; chunks c_begin+1 .. c_begin+PF stay in flight in ring sets 1 .. PF-1, 0
    load_chunk(c_begin, 0);
    store_chunk(0, 0);
#pragma unroll
    for (int i = 1; i <= PF; ++i) load_chunk(c_begin + i, i % PF);
    __syncthreads();

    const int arow = (wm * 32 + l32) * kPA + 16 * lh;
    const int brow = A_BYTES + (wn * 32 + l32) * p.pb + 16 * lh;
    for (int base = c_begin; base < c_end; base += PF) {
#pragma unroll
      for (int u = 0; u < PF; ++u) {
        const int chunk = base + u;
        if (chunk >= c_end) break;   // uniform
        const int buf = (chunk - c_begin) & 1;
        const int8_t* A = lds + buf * STAGE + arow;
        const int8_t* B = lds + buf * STAGE + brow;
        // All LDS reads of this wave's K steps are issued before the first multiply: with one wave per SIMD nothing
        // else hides their latency.
        constexpr int KS = (kKC / 32) / WK;
        if constexpr (S2) {
#pragma unroll
            for (int i = 0; i < KS; ++i) {
                const int ks = wk + i * WK;
                const v4i fa = *reinterpret_cast<const v4i*>(A + 32 * ks);
#pragma unroll
                for (int pl = 0; pl < 4; ++pl) {
                    const int ph_h = pl >> 1, ph_w = pl & 1;
#pragma unroll
                    for (int rs = 0; rs < 2; ++rs) {
                        if (rs == 1 && ph_h == 1) continue;   // kh = 1 is the only tap row on the odd row planes
                        const int kh = ph_h + 2 * rs;
                        // 24 bytes from the dword at or below the first window of this (plane, row shift)
                        const int8_t* src = B + pl * (BN * p.pb) + 32 * ks + ((rs * p.row_pitch) & ~3);
                        const v4i_a4 lo = *reinterpret_cast<const v4i_a4*>(src);
                        const v2i_a4 hi = *reinterpret_cast<const v2i_a4*>(src + 16);
                        const int d[6] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1]};
#pragma unroll
                        for (int cs = 0; cs < 2; ++cs) {
                            if (cs == 1 && ph_w == 1) continue;
                            const int kw = ph_w + 2 * cs;
                            const int sft = (rs ? WQ4 : 0) + cs, j = sft >> 2, sh = sft & 3;
                            v4i bf;
                            if (sh == 0)
                                bf = v4i{d[j], d[j + 1], d[j + 2], d[j + 3]};
                            else
                                bf = v4i{alignbyte(d[j + 1], d[j], sh), alignbyte(d[j + 2], d[j + 1], sh),
                                         alignbyte(d[j + 3], d[j + 2], sh), alignbyte(d[j + 4], d[j + 3], sh)};
                            acc[kh * 3 + kw] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa, bf, acc[kh * 3 + kw], 0, 0, 0);
                        }
                    }
                }
            }
        } else {
        v4i fa[KS];
        int fd[KS][3][6];
#pragma unroll
        for (int i = 0; i < KS; ++i) {
            const int ks = wk + i * WK;
            fa[i] = *reinterpret_cast<const v4i*>(A + 32 * ks);
#pragma unroll
            for (int kh = 0; kh < 3; ++kh) {
                // 24 bytes from the dword at or below this filter row's first window
                const int8_t* src = B + 32 * ks + ((kh * p.row_pitch) & ~3);
                const v4i_a4 lo = *reinterpret_cast<const v4i_a4*>(src);
                const v2i_a4 hi = *reinterpret_cast<const v2i_a4*>(src + 16);
                fd[i][kh][0] = lo[0]; fd[i][kh][1] = lo[1]; fd[i][kh][2] = lo[2]; fd[i][kh][3] = lo[3];
                fd[i][kh][4] = hi[0]; fd[i][kh][5] = hi[1];
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < KS; ++i) {
#pragma unroll
            for (int kh = 0; kh < 3; ++kh) {
                const int r0 = (kh * WQ4) & 3;
                const int* d = fd[i][kh];
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) {
                    const int s = r0 + kw, j = s >> 2, sh = s & 3;
                    v4i bf;
                    if (sh == 0)
                        bf = v4i{d[j], d[j + 1], d[j + 2], d[j + 3]};
                    else
                        bf = v4i{alignbyte(d[j + 1], d[j], sh), alignbyte(d[j + 2], d[j + 1], sh),
                                 alignbyte(d[j + 3], d[j + 2], sh), alignbyte(d[j + 4], d[j + 3], sh)};
                    acc[kh * 3 + kw] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], bf, acc[kh * 3 + kw], 0, 0, 0);
                }
            }
        }
        }
        // chunk+1 sits in ring set (u+1) % PF: it goes to the other LDS buffer and the set is refilled PF chunks ahead
        store_chunk(buf ^ 1, (u + 1) % PF);
        load_chunk(chunk + 1 + PF, (u + 1) % PF);
        __syncthreads();
      }
    }

    // register r of a 32 x 32 tile: row (co) 8*(r/4) + 4*lh + r%4, column (ci) l32; slot = tap*16 + r
    constexpr int SLOTS = kT * 16;
    if constexpr (WK > 1) {
        // ---- combine the eight waves that share a tile, in parallel: every wave owns a share of the slots, hands the
        // other owners theirs through LDS and keeps its own.  The unit of exchange is a quad of slots (the four
        // consecutive registers 4g .. 4g+3 of a tap: one 16-byte LDS access per lane instead of four 4-byte ones);
        // the hand-over area [quad][source wave][lane] for all 36 quads would not fit, so there are two rounds of 18
        // quads, of which waves 0 and 1 own three each and waves 2 .. 7 two each. ----
        static_assert(WK == 8, "the combine below is laid out for eight waves");
        constexpr int QR = SLOTS / 4 / 2;       // quads per round
        auto owner_of = [](int j) { return j < 3 ? 0 : j < 6 ? 1 : 2 + (j - 6) / 2; };   // j: quad inside its round
        auto index_of = [](int j) { return j < 6 ? j % 3 : (j - 6) % 2; };               // position among its owner's quads
        v4i* red4 = reinterpret_cast<v4i*>(lds);
        int* red = reinterpret_cast<int*>(lds);
        int32_t* dst = p.part + ((int64_t)tile * p.splits + split) * SLOTS * kWave + lane;
        v4i own[2 * 3];
#pragma unroll
        for (int rd = 0; rd < 2; ++rd) {
            __syncthreads();   // the staging buffers (or the previous round) are dead from here on
#pragma unroll
            for (int j = 0; j < QR; ++j) {
                const int owner = owner_of(j);
                if (owner != wk) {   // uniform
                    const int Q = rd * QR + j, t = Q / 4, g4 = 4 * (Q % 4);
                    const int srcw = wk < owner ? wk : wk - 1;
                    red4[(j * (WK - 1) + srcw) * kWave + lane] = v4i{acc[t][g4], acc[t][g4 + 1], acc[t][g4 + 2], acc[t][g4 + 3]};
                }
            }
            __syncthreads();
#pragma unroll
            for (int j = 0; j < QR; ++j) {
                if (owner_of(j) != wk) continue;   // uniform
                const int Q = rd * QR + j, t = Q / 4, g4 = 4 * (Q % 4);
                v4i v = {acc[t][g4], acc[t][g4 + 1], acc[t][g4 + 2], acc[t][g4 + 3]};
#pragma unroll
                for (int w = 0; w < WK - 1; ++w) v += red4[(j * (WK - 1) + w) * kWave + lane];
                own[rd * 3 + index_of(j)] = v;
                if (p.splits > 1) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)   // read next by other CUs, not by this one: streaming stores
                        __builtin_nontemporal_store(v[e], &dst[(4 * Q + e) * kWave]);
                }
            }
        }
        if (p.splits > 1) return;
        // Complete tile: dW[co][ci][t] has the 32 ci x 9 taps of one co contiguous (1152 bytes), but a lane holds one
        // ci and a register one (co, t).  The tile is transposed through LDS so that the global stores are row runs.
        __syncthreads();   // everyone is done reading the hand-over area
        constexpr int ROWW = 32 * kT + 1;   // ints per co row in LDS (+1: lanes of a column hit different banks)
#pragma unroll
        for (int Q = 0; Q < SLOTS / 4; ++Q) {
            if (owner_of(Q % QR) != wk) continue;   // uniform
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int t = Q / 4, r = 4 * (Q % 4) + e;
                red[(8 * (r >> 2) + 4 * lh + (r & 3)) * ROWW + l32 * kT + t] = own[(Q / QR) * 3 + index_of(Q % QR)][e];
            }
        }
        __syncthreads();
        const int ncol = min(32, p.Cin - ci0) * kT;   // valid ints of a row
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = wave + WAVES * i, co = co0 + row;
            if (co >= p.Cout) break;
            const float sc = sx * (sc_row[i] / 127.0f);
            const int64_t off = ((int64_t)co * p.Cin + ci0) * kT;
            for (int j = lane; j < ncol; j += kWave) {
                const int v = red[row * ROWW + j];
                store_result(p.dW, off + j, (float)v * sc, p.bf16);
                if (p.acc_out) p.acc_out[off + j] = v;
            }
        }
        return;
    }

    if (p.splits > 1) {
        int32_t* dst = p.part + (((int64_t)tile * p.splits + split) * (WM * WN) + wm * WN + wn) * SLOTS * kWave + lane;
#pragma unroll
        for (int t = 0; t < kT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) dst[(t * 16 + r) * kWave] = acc[t][r];
        return;
    }
    const int ci = ci0 + wn * 32 + l32;
    if (ci >= p.Cin) return;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int co = co0 + wm * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
        if (co < p.Cout) {
            const int64_t off = ((int64_t)co * p.Cin + ci) * kT;
            const float sc = sx * (p.s_chan[co] / 127.0f);
#pragma unroll
            for (int t = 0; t < kT; ++t) {
                store_result(p.dW, off + t, (float)acc[t][r] * sc, p.bf16);
                if (p.acc_out) p.acc_out[off + t] = acc[t][r];
            }
        }
    }
}

// Sum of the K-split partial tiles, then dW = acc * ((s_x/127) * (s_chan[co]/127)), for both kernels of this file
// (the same code serves as a role inside the data-gradient kernel, see dw_tail.h).  With many splits a workgroup
// takes one group of 64 results and its four waves share the splits; with few, every wave takes a group of its own
// and keeps all of its loads in flight - no LDS, no barrier.
__global__ __launch_bounds__(256) void k_dw_reduce(DwTail t) {
    __shared__ int32_t l_sum[4 * kWave];
    if (t.splits > kDwReducePerWave) {
        dw_reduce_role(t, (int)blockIdx.x, l_sum);
        return;
    }
    const int lane = threadIdx.x % kWave;
    const int e = (int)blockIdx.x * 4 + (int)(threadIdx.x / kWave);
    if (e >= t.blocks) return;
    int64_t stride;
    const int32_t* src = dw_tail_source(t, e, lane, stride);
    int32_t v[kDwReducePerWave];
#pragma unroll
    for (int s = 0; s < kDwReducePerWave; ++s) v[s] = src[(int64_t)min(s, t.splits - 1) * stride];
    int32_t a = 0;
#pragma unroll
    for (int s = 0; s < kDwReducePerWave; ++s) a += s < t.splits ? v[s] : 0;
    int co;
    const int64_t off = dw_tail_element(t, e, lane, co);
    if (off < 0) return;
    store_result(t.dW, off, (float)a * ((*t.s_x / 127.0f) * (t.s_chan[co] / 127.0f)), t.bf16);
    if (t.acc_out) t.acc_out[off] = a;
}

// ---------------------------------------------------------------------------------------------
// 1 x 1 filters at unit stride: no tap shifts, so the product is a plain int8 GEMM over the flat axis,
//     acc[co][ci] = sum_f  G[co][f] * X[ci][f] ,
// with both operands staged the same way (rows of 256 + 16 bytes, aligned 16-byte fragment reads).
// A wave owns 64 (co) x 64 (ci): four 32 x 32 tiles, so every fragment it reads feeds two multiplies.
// Same ring, K-split and wave-combine scheme as above.
// ---------------------------------------------------------------------------------------------
// DMA (the eight-wave form): the operands go from global memory straight into LDS (global_load_lds_dwordx4, the 64
// lanes' 16-byte pieces land in 64 consecutive slots), four stage buffers of unpadded 256-byte rows, three stages on
// their way; no staging registers, no LDS stores, one barrier per chunk.  Slot column c of row r holds the row's
// 16-byte column c ^ (r % 16), so that the 16 lanes of a fragment read still fall into different banks.
template <int WM, int WN, int WK, int PF, int CH, bool DMA = false>
__global__ __launch_bounds__(64 * WM * WN * WK) void k_dw11(Dw32Args p) {
    constexpr int WAVES = WM * WN * WK, NT = 64 * WAVES;
    static_assert(WAVES == 4 || WAVES == 8, "four or eight waves");
    constexpr int BM = 64 * WM, BN = 64 * WN;
    constexpr int KCS = CH * kKC;                           // K bytes of a stage: CH chunks between two barriers
    constexpr int PAS = KCS + 16;                           // LDS row pitch of a stage
    constexpr int UPR = KCS / 16;                           // 16-byte units per staged row
    constexpr int UNITS = (BM + BN) * UPR / NT;             // 16-byte units of the two tiles per thread
    constexpr int STAGE = (BM + BN) * PAS;
    static_assert(NT % UPR == 0, "a thread's units all sit in the same 16-byte column of their rows");
    extern __shared__ __align__(16) int8_t lds[];

    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int wk = wave % WK, wn = (wave / WK) % WN, wm = wave / (WK * WN);
    const int l32 = lane & 31, lh = lane >> 5;

    int split, tile;
    if (!dw_block_map(p, split, tile)) return;   // uniform
    const int tn = tile % p.tiles_n, tm = tile / p.tiles_n;
    const int co0 = tm * BM, ci0 = tn * BN;
    const int per = p.nchunks / p.splits, rem = p.nchunks % p.splits;
    const int c_begin = split * per + min(split, rem);
    const int c_end = c_begin + per + (split < rem ? 1 : 0);
    const int c_last = max(c_end - 1, 0);

    // a complete tile is de-quantized here: its scales are requested now, long before they are needed
    float sx = 0.0f, sc_own[WK > 1 ? 8 : 1];
    if (WK > 1 && p.splits == 1) {   // uniform
        sx = *p.s_x;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int q = wk * 8 + e, r = q % 16;
            const int co = co0 + wm * 64 + 32 * (q / 32) + 8 * (r >> 2) + 4 * lh + (r & 3);
            sc_own[e] = p.s_chan[co < p.Cout ? co : 0];
        }
    }

    v16i acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0;

    if constexpr (DMA) {
        static_assert(WM == 1 && WN == 1 && WK == 8 && CH == 1, "the direct-to-LDS form is the eight-wave one");
        typedef __attribute__((address_space(3))) void* lds_ptr;
        constexpr int D = 4;                     // stage buffers
        constexpr int SB = (BM + BN) * kKC;      // bytes of a stage
        // request i of wave w fills rows 16w + 4i .. + 3 of the stage: lane l -> row + l / 16, slot column l % 16
        const int8_t* src[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = 16 * wave + 4 * i + lane / 16;
            const int col = (lane % 16) ^ (row & 15);
            if (row < BM) {   // rows past Cout / Cin recompute row 0 and are never stored
                const int co = co0 + row;
                src[i] = p.g + (int64_t)(co < p.Cout ? co : 0) * p.klen + 16 * col;
            } else {
                const int ci = ci0 + row - BM;
                src[i] = p.x + (int64_t)(ci < p.Cin ? ci : 0) * p.x_chan_pitch + 16 * col;
            }
        }
        // every call issues four requests (past the end the last chunk again, into a buffer nobody reads), so that the
        // count of outstanding requests below is a constant
        auto issue = [&](int chunk, int buf) {
            const int64_t k0 = (int64_t)min(chunk, c_last) * kKC;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                __builtin_amdgcn_global_load_lds(src[i] + k0, (lds_ptr)(lds + buf * SB + (16 * wave + 4 * i) * kKC), 16, 0, 0);
        };
#pragma unroll
        for (int st = 0; st < D - 1; ++st) issue(c_begin + st, st);
        // fragment of K step wk: row l32 (+ 32 t), the row's column 2 wk + lh
        const int fcol = 16 * ((2 * wk + lh) ^ (l32 & 15));
        const int arow = l32 * kKC + fcol, brow = (BM + l32) * kKC + fcol;
        int buf = 0;
        for (int chunk = c_begin; chunk < c_end; ++chunk) {
            asm volatile("s_waitcnt vmcnt(8)" ::: "memory");   // this wave's share of the chunk has landed; two more stages may be on their way
            __builtin_amdgcn_s_barrier();                       // everybody's share has, and the buffer refilled next has been read out
                                                                // (the plain barrier: __syncthreads would wait for the stages on their way too)
            issue(chunk + D - 1, (buf + D - 1) % D);
            const int8_t* A = lds + buf * SB + arow;
            const int8_t* B = lds + buf * SB + brow;
            v4i fa[2], fb[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                fa[t] = *reinterpret_cast<const v4i*>(A + t * 32 * kKC);
                fb[t] = *reinterpret_cast<const v4i*>(B + t * 32 * kKC);
            }
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b) acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[a], fb[b], acc[a][b], 0, 0, 0);
            buf = (buf + 1) % D;
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the requests past the end have landed before LDS is put to other use
    } else {
    // unit u = tid + NT*i -> row u / UPR of the stacked (gradient, activation) tile, 16-byte column u % UPR of the stage;
    // the column - and with it the chunk of the stage the unit belongs to - is the same for all units of a thread
    const int c16 = tid % UPR, sub = c16 / (kKC / 16);
    const int8_t* u_src[UNITS];
    int u_dst[UNITS];
#pragma unroll
    for (int i = 0; i < UNITS; ++i) {
        const int row = (tid + NT * i) / UPR;
        if (row < BM) {   // rows past Cout / Cin recompute row 0 and are never stored
            const int co = co0 + row;
            u_src[i] = p.g + (int64_t)(co < p.Cout ? co : 0) * p.klen + 16 * (c16 % (kKC / 16));
        } else {
            const int ci = ci0 + row - BM;
            u_src[i] = p.x + (int64_t)(ci < p.Cin ? ci : 0) * p.x_chan_pitch + 16 * (c16 % (kKC / 16));
        }
        u_dst[i] = row * PAS + 16 * c16;
    }
    // Every call issues the same loads (past the end the last chunk is fetched again, which the caches absorb, and
    // never multiplied): only then can the compiler count the loads in flight and wait for exactly the oldest set.
    v4i ring[PF][UNITS];
    auto load_stage = [&](int chunk, int set) {   // chunk: the first of the stage
        const int64_t k0 = (int64_t)min(chunk + sub, c_last) * kKC;
#pragma unroll
        for (int i = 0; i < UNITS; ++i) ring[set][i] = *reinterpret_cast<const v4i*>(u_src[i] + k0);
        __builtin_amdgcn_sched_barrier(0);   // keep the sets in program order
    };
    auto store_stage = [&](int buf, int set) {
#pragma unroll
        for (int i = 0; i < UNITS; ++i) *reinterpret_cast<v4i*>(lds + buf * STAGE + u_dst[i]) = ring[set][i];
    };

    load_stage(c_begin, 0);
    store_stage(0, 0);
#pragma unroll
    for (int i = 1; i <= PF; ++i) load_stage(c_begin + i * CH, i % PF);
    __syncthreads();

    const int arow = (wm * 64 + l32) * PAS + 16 * lh;
    const int brow = (BM + wn * 64 + l32) * PAS + 16 * lh;
    int buf = 0;
    for (int base = c_begin; base < c_end; base += PF * CH) {
#pragma unroll
      for (int u = 0; u < PF; ++u) {
        const int chunk = base + u * CH;
        if (chunk >= c_end) break;   // uniform
        const int8_t* A = lds + buf * STAGE + arow;
        const int8_t* B = lds + buf * STAGE + brow;
        constexpr int KS = (kKC / 32) / WK;
        v4i fa[CH][KS][2], fb[CH][KS][2];
#pragma unroll
        for (int j = 0; j < CH; ++j)
#pragma unroll
            for (int i = 0; i < KS; ++i) {
                const int ks = wk + i * WK;
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    fa[j][i][t] = *reinterpret_cast<const v4i*>(A + t * 32 * PAS + j * kKC + 32 * ks);
                    fb[j][i][t] = *reinterpret_cast<const v4i*>(B + t * 32 * PAS + j * kKC + 32 * ks);
                }
            }
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            if (j > 0 && chunk + j >= c_end) break;   // uniform: the stage's later chunks lie past this split's share
#pragma unroll
            for (int i = 0; i < KS; ++i)
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[j][i][a], fb[j][i][b], acc[a][b], 0, 0, 0);
        }
        store_stage(buf ^ 1, (u + 1) % PF);
        load_stage(chunk + (1 + PF) * CH, (u + 1) % PF);
        buf ^= 1;
        __syncthreads();
      }
    }
    }

    // slot q = (a*2 + b)*16 + r: tile (a, b) of the wave, register r -> row (co) 32a + 8*(r/4) + 4*lh + r%4, column (ci) 32b + l32
    constexpr int SLOTS = 64;
    v4i own[2];   // WK = 8: the two quads of slots (four consecutive registers of one tile) this wave owns
    if constexpr (WK > 1) {
        // parallel combine of the eight waves as in k_dw32, in one round: 16 quads, two per wave,
        // hand-over area [quad][source wave][lane] of 16-byte entries
        static_assert(WK == 8, "the combine below is laid out for eight waves");
        v4i* red4 = reinterpret_cast<v4i*>(lds);
        __syncthreads();   // the staging buffers are dead from here on
#pragma unroll
        for (int Q = 0; Q < SLOTS / 4; ++Q) {
            const int owner = Q / 2;
            if (owner != wk) {   // uniform
                const int srcw = wk < owner ? wk : wk - 1;
                const int g4 = 4 * (Q % 4);
                const v16i& tl = acc[Q / 8][(Q / 4) % 2];
                red4[(Q * (WK - 1) + srcw) * kWave + lane] = v4i{tl[g4], tl[g4 + 1], tl[g4 + 2], tl[g4 + 3]};
            }
        }
        __syncthreads();
#pragma unroll
        for (int Q = 0; Q < SLOTS / 4; ++Q) {
            if (Q / 2 != wk) continue;   // uniform
            const int g4 = 4 * (Q % 4);
            const v16i& tl = acc[Q / 8][(Q / 4) % 2];
            v4i v = {tl[g4], tl[g4 + 1], tl[g4 + 2], tl[g4 + 3]};
#pragma unroll
            for (int w = 0; w < WK - 1; ++w) v += red4[(Q * (WK - 1) + w) * kWave + lane];
            own[Q % 2] = v;
        }
    }
    int32_t* dst = p.part + (((int64_t)tile * p.splits + split) * (WM * WN) + wm * WN + wn) * SLOTS * kWave + lane;
    if (WK == 1 && p.splits == 1) sx = *p.s_x;
    sx = sx / 127.0f;
#pragma unroll
    for (int q = 0; q < SLOTS; ++q) {
        if (WK > 1 && q / 8 != wk) continue;   // uniform: not this wave's slot
        const int v = WK > 1 ? own[(q / 4) % 2][q % 4] : acc[q / 32][(q / 16) % 2][q % 16];
        if (p.splits > 1) {
            __builtin_nontemporal_store(v, &dst[q * kWave]);   // read next by other CUs, not by this one
        } else {
            const int r = q % 16;
            const int co = co0 + wm * 64 + 32 * (q / 32) + 8 * (r >> 2) + 4 * lh + (r & 3);
            const int ci = ci0 + wn * 64 + 32 * ((q / 16) % 2) + l32;
            if (co < p.Cout && ci < p.Cin) {
                const int64_t off = (int64_t)co * p.Cin + ci;   // 32 lanes = 32 consecutive ci: 128-byte runs
                const float sc = WK > 1 ? sc_own[q % 8] : p.s_chan[co];
                store_result(p.dW, off, (float)v * (sx * (sc / 127.0f)), p.bf16);
                if (p.acc_out) p.acc_out[off] = v;
            }
        }
    }
}

struct Plan32 {
    bool ok;
    bool k11;             // 1 x 1 filter: the plain GEMM kernel
    bool s2;              // 3 x 3 filter at stride 2: four stride-phase planes per input channel
    int wm, wn, wk, splits, tiles_m, tiles_n, nchunks, pb, b_units, ch;
    int bands_m, bands_n, band_m, band_n;   // rectangles of the tile grid per K split when there are 1, 2 or 4 splits (else 0)
    int64_t blocks;       // workgroups of the launch
    size_t lds_bytes;
    int64_t part_slots;   // int32 entries of one split's partial tiles
};

// Rectangles per split for 1, 2 or 4 splits (8, 4 or 2 XCDs share a split): the cut of the tile grid that makes an
// XCD touch the fewest operand rows, rows of the two operands weighted by their tile heights.
void choose_bands(Plan32& pl, int bm, int bn) {
    pl.bands_m = pl.bands_n = pl.band_m = pl.band_n = 0;
    pl.blocks = (int64_t)pl.tiles_m * pl.tiles_n * pl.splits;
    if (pl.splits != 1 && pl.splits != 2 && pl.splits != 4) return;
    const int rects = kXcd / pl.splits;
    int64_t best = -1;
    for (int rm = 1; rm <= rects; rm *= 2) {
        const int rn = rects / rm;
        if (rm > pl.tiles_m || rn > pl.tiles_n) continue;
        const int64_t hm = ceil_div(pl.tiles_m, rm), hn = ceil_div(pl.tiles_n, rn);
        const int64_t rows = hm * bm + hn * bn;
        if (best < 0 || rows < best) { best = rows; pl.bands_m = rm; pl.bands_n = rn; pl.band_m = (int)hm; pl.band_n = (int)hn; }
    }
    if (best < 0) { pl.bands_m = pl.bands_n = 0; return; }
    pl.blocks = (int64_t)kXcd * pl.band_m * pl.band_n;
}

Plan32 make_plan32(const daq_conv_desc& d) {
    Plan32 pl{};
    if (d.groups != 1) return pl;
    const bool unit = d.strideH == 1 && d.strideW == 1 && d.dilH == 1 && d.dilW == 1;
    // a 1 x 1 filter pairs gradient position f with byte f of the activation's first stride-phase plane whatever the
    // stride (and dilation means nothing), so the plain GEMM serves strided shortcuts too
    const bool k33 = unit && d.kH == 3 && d.kW == 3, k11 = d.kH == 1 && d.kW == 1;
    const bool k33s2 = d.kH == 3 && d.kW == 3 && d.strideH == 2 && d.strideW == 2 && d.dilH == 1 && d.dilW == 1;
    if (!k33 && !k11 && !k33s2) return pl;
    daq_layout Lg, Lx;
    if (daq_layout_vq(&d, &Lg) != DAQ_OK || daq_layout_qx_cnhw(&d, &Lx) != DAQ_OK) return pl;
    if (Lg.bytes >= ((int64_t)1 << 32) || Lx.bytes >= ((int64_t)1 << 32)) return pl;   // 32-bit per-lane offsets
    pl.nchunks = (int)(Lg.plane_pitch / kKC);
    if (k11) {
        // plain GEMM: 64 x 64 per wave; 128 x 128 per workgroup when that alone fills the chip, else eight waves on one
        // 64 x 64 tile with K split among them and across workgroups
        pl.k11 = true;
        const int64_t t128 = ceil_div(d.Cout, 128) * ceil_div(d.Cin, 128);
        if (t128 >= 256) { pl.wm = 2; pl.wn = 2; pl.wk = 1; }
        else { pl.wm = 1; pl.wn = 1; pl.wk = 8; }
        pl.tiles_m = (int)ceil_div(d.Cout, 64 * pl.wm);
        pl.tiles_n = (int)ceil_div(d.Cin, 64 * pl.wn);
        const int64_t tiles = (int64_t)pl.tiles_m * pl.tiles_n;
        int64_t s = ceil_div(256, tiles);
        s = std::min<int64_t>(s, std::max(1, pl.nchunks / 2));
        pl.splits = (int)std::max<int64_t>(1, s);
        // One chunk per LDS stage.  (Two chunks per barrier were measured on the late ResNet-50 layers: the K loop of a
        // workgroup - 13 chunks of 32 KiB in 7 us on every CU at once, bound by the staging through registers and LDS and
        // its two waits per chunk - gets a quarter shorter per byte, and the first stage arrives that much later.)
        pl.ch = 1;
        const size_t stage = (size_t)64 * (pl.wm + pl.wn) * (pl.ch * kKC + 16);
        pl.lds_bytes = std::max<size_t>(pl.wk > 1 ? (size_t)4 * 128 * kKC : 2 * stage, pl.wk > 1 ? (size_t)(pl.wk - 1) * 64 * kWave * 4 : 0);   // staging (four unpadded stages in the direct-to-LDS form); one-round combine
        pl.part_slots = tiles * pl.wm * pl.wn * 64 * kWave;
        choose_bands(pl, 64 * pl.wm, 64 * pl.wn);
        pl.ok = true;
        return pl;
    }
    if (k33s2) {
        // the strided form relies on the slot geometry the two operands share and on the four phase planes of a channel
        if (Lx.phases_h != 2 || Lx.phases_w != 2 || Lx.row_pitch != Lg.row_pitch || Lx.img_rows != Lg.img_rows ||
            Lx.lead != Lg.lead || Lx.chan_pitch != 4 * Lx.plane_pitch)
            return pl;
        pl.s2 = true;
    }
    // bytes of an activation row a chunk needs: its own 256 plus the largest tap offset, plus the bytes the
    // six-dword reads of the last K step touch beyond that
    const int need = kKC + (pl.s2 ? 1 : 2) * Lx.row_pitch + 2 + 8;
    pl.b_units = (int)ceil_div(need, 16);
    pl.pb = 16 * pl.b_units + 4;              // pitch/4 odd: the 32 rows of a fragment read fall into 32 different banks
    const int64_t t64 = ceil_div(d.Cout, 64) * ceil_div(d.Cin, 64);
    if (t64 >= 256 && !pl.s2) { pl.wm = 2; pl.wn = 2; pl.wk = 1; }
    else { pl.wm = 1; pl.wn = 1; pl.wk = 8; }   // eight waves: two per SIMD, so that one's LDS phase overlaps the other's MFMAs
    const int bm = 32 * pl.wm, bn = 32 * pl.wn;
    if (pl.s2 ? 4 * bn * pl.b_units > 5 * 512 : (int64_t)bn * pl.b_units > 4 * pl.wn * 256) return pl;   // staging registers of the activation tile (B_MAX * threads)
    pl.tiles_m = (int)ceil_div(d.Cout, bm);
    pl.tiles_n = (int)ceil_div(d.Cin, bn);
    const int64_t tiles = (int64_t)pl.tiles_m * pl.tiles_n;
    int64_t s = ceil_div(256, tiles);
    s = std::min<int64_t>(s, std::max(1, pl.nchunks / 2));
    pl.splits = (int)std::max<int64_t>(1, s);
    const size_t stage = (size_t)bm * kPA + (size_t)(pl.s2 ? 4 : 1) * bn * pl.pb;
    // hand-over area of the parallel combine: [owner][source][slot][lane]
    const int rounds = pl.wk > 4 ? 2 : 1;
    pl.lds_bytes = std::max<size_t>(2 * stage, pl.wk > 1 ? (size_t)(pl.wk - 1) * kT * 16 * kWave * 4 / rounds : 0);
    if (pl.lds_bytes > 150 * 1024) return pl;
    pl.part_slots = tiles * pl.wm * pl.wn * kT * 16 * kWave;
    choose_bands(pl, bm, bn);
    pl.ok = true;
    return pl;
}

template <int WM, int WN, int WK, int PF, bool S2 = false>
daq_status launch32(const Plan32& pl, const Dw32Args& a, int wq4, hipStream_t st) {
    const dim3 grid((unsigned)pl.blocks);
#define DAQ_DW32_CASE(Q)                                                                                          \
    if (wq4 == Q) {                                                                                               \
        auto kern = k_dw32<Q, WM, WN, WK, PF, S2>;                                                                    \
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,                    \
                                (int)pl.lds_bytes) != hipSuccess)                                                 \
            return DAQ_ERR_HIP;                                                                                   \
        DAQ_LAUNCH("conv_bwd_filter_dw32", st, hipLaunchKernelGGL(kern, grid, dim3(64 * WM * WN * WK), pl.lds_bytes, st, a)); \
        return DAQ_OK;                                                                                            \
    }
    DAQ_DW32_CASE(0) DAQ_DW32_CASE(1) DAQ_DW32_CASE(2) DAQ_DW32_CASE(3)
#undef DAQ_DW32_CASE
    return DAQ_ERR_UNSUPPORTED;
}

}  // namespace

bool bwd_filter_lds_supported(const daq_conv_desc& d) { return make_plan32(d).ok; }

size_t bwd_filter_lds_ws_bytes(const daq_conv_desc& d) {
    const Plan32 pl = make_plan32(d);
    if (!pl.ok || pl.splits == 1) return 0;
    return (size_t)round_up(pl.part_slots * pl.splits * 4, 256);
}

daq_status conv_bwd_filter_lds(const daq_conv_desc& d, const int8_t* qx, const float* s_x, const int8_t* vq,
                               const float* s_chan, float* dW, int32_t* acc, void* ws, hipStream_t st, DwTail* defer, bool bf16) {
    if (defer) defer->blocks = 0;
    const Plan32 pl = make_plan32(d);
    if (!pl.ok) return DAQ_ERR_UNSUPPORTED;
    daq_layout Lx, Lg;
    if (daq_layout_qx_cnhw(&d, &Lx) != DAQ_OK || daq_layout_vq(&d, &Lg) != DAQ_OK) return DAQ_ERR_INVALID_ARG;
    Dw32Args a{};
    a.g = vq;
    a.x = qx;
    a.klen = Lg.plane_pitch;
    a.x_chan_pitch = Lx.chan_pitch;
    a.x_plane_pitch = Lx.plane_pitch;
    a.Cout = d.Cout;
    a.Cin = d.Cin;
    a.row_pitch = Lx.row_pitch;
    a.pb = pl.pb;
    a.b_units = pl.b_units;
    a.nchunks = pl.nchunks;
    a.splits = pl.splits;
    a.tiles_n = pl.tiles_n;
    a.tiles_m = pl.tiles_m;
    a.bands_m = pl.bands_m; a.bands_n = pl.bands_n; a.band_m = pl.band_m; a.band_n = pl.band_n;
    a.part = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(ws) + 256);
    a.s_x = s_x;
    a.s_chan = s_chan;
    a.dW = dW;
    a.acc_out = acc;
    a.bf16 = bf16 ? 1 : 0;
    const int wq4 = Lx.row_pitch & 3;
    if (pl.k11) {
        const dim3 grid((unsigned)pl.blocks);
        if (pl.wk == 1) {
            auto kern = k_dw11<2, 2, 1, 1, 1>;
            if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.lds_bytes) != hipSuccess)
                return DAQ_ERR_HIP;
            DAQ_LAUNCH("conv_bwd_filter_dw11", st, hipLaunchKernelGGL(kern, grid, dim3(256), pl.lds_bytes, st, a));
        } else {
            auto kern = k_dw11<1, 1, 8, 3, 1, true>;
            if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.lds_bytes) != hipSuccess)
                return DAQ_ERR_HIP;
            DAQ_LAUNCH("conv_bwd_filter_dw11", st, hipLaunchKernelGGL(kern, grid, dim3(512), pl.lds_bytes, st, a));
        }
        if (pl.splits > 1 && defer && dw_tail_worthwhile((int)(pl.part_slots / kWave), pl.splits))
            *defer = DwTail{a.part, (int)(pl.part_slots / kWave), pl.splits, pl.tiles_n, pl.wm, pl.wn, d.Cout, d.Cin, 1, s_x, s_chan, dW, acc, bf16 ? 1 : 0};
        else if (pl.splits > 1) {
            const DwTail t{a.part, (int)(pl.part_slots / kWave), pl.splits, pl.tiles_n, pl.wm, pl.wn, d.Cout, d.Cin, 1, s_x, s_chan, dW, acc, bf16 ? 1 : 0};
            const unsigned blocks = pl.splits > kDwReducePerWave ? (unsigned)t.blocks : (unsigned)ceil_div(t.blocks, 4);
            DAQ_LAUNCH("dw_reduce", st, hipLaunchKernelGGL(k_dw_reduce, dim3(blocks), dim3(256), 0, st, t));
        }
        return DAQ_OK;
    }
    const daq_status rc = pl.s2 ? launch32<1, 1, 8, 2, true>(pl, a, wq4, st)
                          : pl.wk == 1 ? launch32<2, 2, 1, 1>(pl, a, wq4, st) : launch32<1, 1, 8, 3>(pl, a, wq4, st);
    if (rc != DAQ_OK) return rc;
    if (pl.splits > 1 && defer && dw_tail_worthwhile((int)(pl.part_slots / kWave), pl.splits)) {
        *defer = DwTail{a.part, (int)(pl.part_slots / kWave), pl.splits, pl.tiles_n, pl.wm, pl.wn, d.Cout, d.Cin, 9, s_x, s_chan, dW, acc, bf16 ? 1 : 0};
    } else if (pl.splits > 1) {
        const DwTail t{a.part, (int)(pl.part_slots / kWave), pl.splits, pl.tiles_n, pl.wm, pl.wn, d.Cout, d.Cin, 9, s_x, s_chan, dW, acc, bf16 ? 1 : 0};
        const unsigned blocks = pl.splits > kDwReducePerWave ? (unsigned)t.blocks : (unsigned)ceil_div(t.blocks, 4);
        DAQ_LAUNCH("dw_reduce", st, hipLaunchKernelGGL(k_dw_reduce, dim3(blocks), dim3(256), 0, st, t));
    }
    return DAQ_OK;
}

}  // namespace daq
