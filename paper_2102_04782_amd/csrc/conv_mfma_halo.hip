// Channel-contracting int8 implicit GEMM, halo-tile form: the data gradient q(G_X) = q(G) (.) q(W)
// (Eq. "gx") for strides 1 and 2, and the unit-stride forward convolution.
//
//     C[row channel][pixel] = sum over (tap, k)  Wp[tap][row][k] * P[src_pixel(pixel, tap)][k]
//
// A workgroup owns NI images x (TH x TW) destination pixels (<= 256) and 64 or 128 row channels.
// Per 64-byte chunk of the contraction axis it stages the SOURCE WINDOW of its tile in LDS once -
// (TH + reach) x (TW + reach) pixel slots of 64 channel bytes - and every filter tap reads that
// window at a shifted slot, so no pixel is staged more than once and the loop over the taps has no
// LDS writes and no barrier.  The filter operand never goes through LDS: it is stored in fragment
// order (see daq_wpack_layout), so a wave fetches each 32-row x 32-byte tile as one contiguous KiB
// straight into the registers the MFMA reads, one step ahead.  The window of the next chunk is
// fetched while the taps of the current one run and is written to the other LDS buffer at the
// chunk's last tap: one barrier per chunk.
//
// Stride 2 (data gradient only): destination pixels are split by parity (h % 2, w % 2).  Pixels of
// one parity class see the same subset of taps, each at a unit-stride position of the source, so a
// workgroup handles one class and issues only the taps that are live for it - no multiplies by
// stride-skipped zeros.
#include <algorithm>

#include "daq_internal.h"
#include "dw_tail.h"

namespace daq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kPxWg = 256;         // destination pixels per workgroup (128 in the small-tile form of 1 x 1 filters)
constexpr int kKc = 64;            // contraction bytes per step (two MFMA K-steps of 32)
constexpr int kPitch = kKc + 16;   // LDS pitch of a window slot: eight consecutive slots cover all banks
constexpr int kMaxTaps = 49;
constexpr int kMaxUnits = 8;       // 16-byte units of the window a thread stages: up to 512 slots
constexpr int kMaxPhases = 4;
constexpr int kRingA = 4;          // filter tiles are requested kRingA - 1 steps ahead of their use
constexpr uint32_t kOob = 0x80000000u;  // a buffer offset past every extent: such a load returns zeros

struct HaloArgs {
    const int8_t* src;    // pixel operand, NHWC [N][Hs][Ws][cp]
    const int8_t* wfrag;  // filter operand in fragment order
    uint32_t src_bytes, wfrag_bytes;
    int N, Hs, Ws, cp;
    int Hd, Wd;
    int Crow, RB, T;      // result channels, 32-row blocks of the filter copy, kH*kW
    int stride;           // 1, or 2 (parity classes)
    int TH, TW, NI;       // destination tile, in pixels of one parity class
    int SH, SW;           // source window per image (the largest over the classes)
    int tiles_h, tiles_w, groups;
    int units;            // 16-byte window units per thread
    int double_buffer;    // more than one contraction chunk: two window buffers
    int zfill;            // stride 2, only parity class (0, 0) has taps: its workgroups also write the zeros of the other three
    // per parity class: live taps, window origin relative to the tile's first pixel
    int ph_taps[kMaxPhases], ph_org_h[kMaxPhases], ph_org_w[kMaxPhases];
    // 32-bit entries: a uniform index then costs a scalar load, not a vector-memory round trip
    int tap_slot[kMaxPhases][kMaxTaps];  // slot offset a tap adds inside the window
    int tap_id[kMaxPhases][kMaxTaps];    // kh*kW + kw of the tap
    FastDiv div_tw, div_thw, div_sw, div_si, div_tiles_w, div_tiles_hw, div_ptiles;
    const float* s_a;
    const float* s_b;
    float* out;           // fp32 [N][Crow][Hd][Wd]
    int32_t* acc_out;
    DwTail tail;          // tail.blocks > 0: that many workgroups behind the first main_blocks finish a deferred filter
    int main_blocks;      // gradient instead (they are dispatched last and fill the slots this kernel's own tiles leave)
    int bf16;             // the result is stored as bfloat16 (round to nearest even) instead of fp32
    int nt;               // the result is large: streaming stores, so that it does not push the next kernels' operands out of the caches
};

__device__ __forceinline__ v4i buffer_load16(__amdgpu_buffer_rsrc_t rsrc, uint32_t voffset, uint32_t soffset) {
    return __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voffset, (int)soffset, 0);
}

// WR = waves along the row (output channel) axis, WAVES = waves per workgroup.  (1, 4): 64 rows x 256 pixels with
// 64 x 64 wave tiles.  (2, 4): 128 rows x 256 pixels with 64 x 128 wave tiles.  (2, 8): the same workgroup tile with
// 64 x 64 wave tiles on eight waves - two per SIMD, so that the LDS reads of one overlap the multiplies of the other.
// DB = the contraction axis has more than one 64-byte chunk (two window buffers, restaged per chunk).
// ST = stride (1 or 2): with one parity class its tables are indexed with constants.
// TAPS > 0 (unit stride; TAPS = 1 also stride 2 with a single live parity class): the number of filter taps is this constant.  The loop over the taps of a chunk is
// then unrolled, the ring of filter tiles has one slot per tap (slot = tap, so each tile is requested TAPS - 1
// steps before its use), the tap tables are read once, and the pixel fragments of the next tap are read from LDS
// before the multiplies of the current one: with a single wave per SIMD nothing else hides those latencies.
// NX = 32-row blocks of a wave that can hold result rows: 1 for results of at most 32 channels (the data gradient of a
// network's first layer), whose second block would only multiply zeros - dynamic-tap form on 64-row tiles only.
// PX = destination pixels per workgroup: 128 (a wave then owns 64 rows x 32 pixels) for 1 x 1 layers with so few
// pixels that 256-pixel tiles would leave CUs without a workgroup.
template <int WR, bool DB, int ST, int WAVES, int TAPS = 0, int NX = 2, int PX = kPxWg>
__global__ __launch_bounds__(64 * WAVES, (TAPS == 1 || NX == 1 || PX < kPxWg) ? 2 : 1) void k_conv_halo(HaloArgs p) {
    constexpr int ROWS = 64 * WR;
    constexpr int WPX = WAVES / WR;
    constexpr int SPT = 16 * WAVES;   // window slots one pass of the workgroup stages (four lanes per slot)
    constexpr int PXW = PX / WPX;
    constexpr int BF = PXW / 32;
    extern __shared__ __align__(16) int8_t lds[];   // one or two window buffers of S slots

    if (p.tail.blocks > 0 && (int)blockIdx.x >= p.main_blocks) {   // uniform
        dw_reduce_role(p.tail, (int)blockIdx.x - p.main_blocks, reinterpret_cast<int32_t*>(lds));
        return;
    }
    const uint32_t bid = blockIdx.x;
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int l32 = lane & 31, lh = lane >> 5;
    const int wr = wave % WR, wp = wave / WR;
    // block -> (row tile, parity class, image group, tile row, tile column)
    const int per_phase = p.groups * p.tiles_h * p.tiles_w;
    const int ptiles = (ST > 1 && !p.zfill) ? ((per_phase + 7) & ~7) * (ST * ST) : per_phase;
    const int tr = (int)fdiv(bid, p.div_ptiles);
    int tp = (int)bid - tr * ptiles;
    int phase = 0;
    if (ST > 1 && !p.zfill) {
        // The four parity classes of a tile interleave in memory (every other pixel of every other row), so each of them
        // writes partial cache lines.  Their workgroups sit 8 blocks apart in groups of 32: same XCD (block i runs on
        // XCD i % 8), dispatched together, and the partial lines meet in one L2 instead of going to memory one by one.
        const int g8 = tp >> 5, r = tp & 31;
        phase = r >> 3;
        tp = g8 * 8 + (r & 7);
        if (tp >= per_phase) return;   // uniform: padding of the last group of eight tiles
    }
    const int pa = phase / ST, pb = phase % ST;
    const int grp = (int)fdiv((uint32_t)tp, p.div_tiles_hw);
    const int trem = tp - grp * p.tiles_h * p.tiles_w;
    const int tih = (int)fdiv((uint32_t)trem, p.div_tiles_w);
    const int tiw = trem - tih * p.tiles_w;
    const int row0 = tr * ROWS;
    const int n0 = grp * p.NI, h0 = tih * p.TH, w0 = tiw * p.TW;
    const int SI = p.SH * p.SW, S = p.NI * SI;
    const int halo_bytes = S * kPitch;
    const int nkc = (p.cp + kKc - 1) / kKc;
    const int taps = p.ph_taps[phase];
    const int NS = nkc * taps;
    const int org_h = p.ph_org_h[phase], org_w = p.ph_org_w[phase];

    const __amdgpu_buffer_rsrc_t rs_src = __builtin_amdgcn_make_buffer_rsrc((void*)p.src, 0, (int)p.src_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc((void*)p.wfrag, 0, (int)p.wfrag_bytes, 0x00020000);
    // the de-quantization factor is requested here, not in the epilogue, where its latency would show
    const float scale = (*p.s_a / 127.0f) * (*p.s_b / 127.0f);

    // ---- window staging: unit i of a thread is chunk (tid & 3) of slot (tid >> 2) + SPT*i ----
    const int sc = tid & 3;
    uint32_t hoff[kMaxUnits];
#pragma unroll
    for (int i = 0; i < kMaxUnits; ++i) {
        hoff[i] = kOob;
        if (i < p.units) {   // uniform
            const int slot = (tid >> 2) + SPT * i;
            const int img = (int)fdiv((uint32_t)slot, p.div_si);
            const int rem = slot - img * SI;
            const int r = (int)fdiv((uint32_t)rem, p.div_sw);
            const int c = rem - r * p.SW;
            const int n = n0 + img, hs = h0 + org_h + r, ws = w0 + org_w + c;
            const bool ok = slot < S && n < p.N && (unsigned)hs < (unsigned)p.Hs && (unsigned)ws < (unsigned)p.Ws;
            if (ok) hoff[i] = (uint32_t)(((n * p.Hs + hs) * p.Ws + ws) * p.cp + 16 * sc);
        }
    }
    v4i rh[kMaxUnits];
    auto fetch_halo = [&](int kci) {
        const bool kok = kci < nkc && kci * kKc + 16 * sc < p.cp;
#pragma unroll
        for (int i = 0; i < kMaxUnits; ++i)
            if (i < p.units) rh[i] = buffer_load16(rs_src, kok ? hoff[i] : kOob, (uint32_t)(kci * kKc));
    };
    auto stage_halo = [&](int buf) {
        int8_t* H = lds + buf * halo_bytes;
#pragma unroll
        for (int i = 0; i < kMaxUnits; ++i) {
            const int slot = (tid >> 2) + SPT * i;
            if (i < p.units && slot < S) *reinterpret_cast<v4i*>(H + slot * kPitch + 16 * sc) = rh[i];
        }
    };

    // ---- filter fragments: tile (x, sub) of this wave is 1 KiB at ((row block)*2 + sub)*1024, lane*16 inside ----
    uint32_t aoff[2][2];
#pragma unroll
    for (int x = 0; x < NX; ++x)
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const int rb = (row0 + wr * 64) / 32 + x;
            aoff[x][sub] = rb < p.RB ? (uint32_t)((rb * 2 + sub) * 1024 + lane * 16) : kOob;
        }
    v4i ra[kRingA][2][2];   // [ring slot][x][sub]
    int f_j = 0, f_kc = 0, f_s = 0;
    auto fetch_a = [&](int slot) {
        const bool live = f_s < NS;
        const int id = p.tap_id[phase][live ? f_j : 0];
        // a dead prefetch is sent out of range through the VECTOR offset, the one the hardware checks against the extent
        const uint32_t base = live ? (uint32_t)(((f_kc * p.T + id) * p.RB) * 2048) : 0u;
#pragma unroll
        for (int x = 0; x < NX; ++x)
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) ra[slot][x][sub] = buffer_load16(rs_w, live ? aoff[x][sub] : kOob, base);
        ++f_s;
        if (++f_j == taps) { f_j = 0; ++f_kc; }
    };

    // ---- pixel fragments: destination pixel q of the tile -> slot of its window origin ----
    int bslot[BF];
#pragma unroll
    for (int y = 0; y < BF; ++y) {
        const int q = wp * PXW + 32 * y + l32;
        const int img = (int)fdiv((uint32_t)q, p.div_thw);
        const int rem = q - img * p.TH * p.TW;
        const int th = (int)fdiv((uint32_t)rem, p.div_tw);
        const int tw = rem - th * p.TW;
        bslot[y] = (img < p.NI) ? img * SI + th * p.SW + tw : 0;
    }

    v16i acc[2][BF];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < BF; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0;

    if constexpr (TAPS == 1) {
        // 1 x 1 filters: a step is a chunk, and every chunk needs a new window.  With the window requested only one
        // step ahead each chunk would wait out a full memory latency; here window registers and filter tiles both
        // sit in rings of kRing1 chunks (slot = chunk % kRing1), requested kRing1 - 1 chunks before their use.
        constexpr int kRing1 = 4, kU1 = PX / 64;   // kU1: 16-byte window units per thread (no halo: at most PX slots)
        v4i ra1[kRing1][2][2], rw[kRing1][kU1];
        auto fetch_1 = [&](int slot, int kc) {
            const bool live = kc < nkc;
            const uint32_t base = live ? (uint32_t)((kc * p.RB) * 2048) : 0u;
#pragma unroll
            for (int x = 0; x < NX; ++x)
#pragma unroll
                for (int sub = 0; sub < 2; ++sub) ra1[slot][x][sub] = buffer_load16(rs_w, live ? aoff[x][sub] : kOob, base);
            const bool kok = live && kc * kKc + 16 * sc < p.cp;
#pragma unroll
            for (int i = 0; i < kU1; ++i)
                if (i < p.units) rw[slot][i] = buffer_load16(rs_src, kok ? hoff[i] : kOob, (uint32_t)(kc * kKc));
        };
        auto stage_1 = [&](int buf, int slot) {
            int8_t* H = lds + buf * halo_bytes;
#pragma unroll
            for (int i = 0; i < kU1; ++i) {
                const int sl = (tid >> 2) + SPT * i;
                if (i < p.units && sl < S) *reinterpret_cast<v4i*>(H + sl * kPitch + 16 * sc) = rw[slot][i];
            }
        };
        int bbyte[BF];
#pragma unroll
        for (int y = 0; y < BF; ++y) bbyte[y] = bslot[y] * kPitch + 16 * lh;
#pragma unroll
        for (int c = 0; c < kRing1 - 1; ++c) fetch_1(c, c);
        stage_1(0, 0);
        __syncthreads();
        for (int base = 0; base < nkc; base += kRing1) {
#pragma unroll
            for (int u = 0; u < kRing1; ++u) {
                const int kc = base + u;
                if (kc >= nkc) break;   // uniform
                fetch_1((u + kRing1 - 1) % kRing1, kc + kRing1 - 1);
                const int8_t* H = lds + (kc & 1) * halo_bytes;
#pragma unroll
                for (int sub = 0; sub < 2; ++sub) {
                    v4i b[BF];
#pragma unroll
                    for (int y = 0; y < BF; ++y) b[y] = *reinterpret_cast<const v4i*>(H + bbyte[y] + 32 * sub);
#pragma unroll
                    for (int x = 0; x < NX; ++x)
#pragma unroll
                        for (int y = 0; y < BF; ++y)
                            acc[x][y] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ra1[u][x][sub], b[y], acc[x][y], 0, 0, 0);
                }
                if (kc + 1 < nkc) {
                    stage_1((kc + 1) & 1, (u + 1) % kRing1);
                    __syncthreads();
                }
            }
        }
    } else if constexpr (TAPS > 0) {
        // tap tables: loop invariant, indexed with constants after unrolling
        int t_id[TAPS], t_off[TAPS];
#pragma unroll
        for (int t = 0; t < TAPS; ++t) {
            t_id[t] = p.tap_id[0][t];
            t_off[t] = p.tap_slot[0][t] * kPitch;
        }
        int bbyte[BF];
#pragma unroll
        for (int y = 0; y < BF; ++y) bbyte[y] = bslot[y] * kPitch + 16 * lh;
        v4i rt[TAPS][2][2];   // [tap][x][sub]
        auto fetch_t = [&](int t, int kc) {
            const bool live = kc < nkc;
            const uint32_t base = live ? (uint32_t)(((kc * p.T + t_id[t]) * p.RB) * 2048) : 0u;
#pragma unroll
            for (int x = 0; x < NX; ++x)
#pragma unroll
                for (int sub = 0; sub < 2; ++sub) rt[t][x][sub] = buffer_load16(rs_w, live ? aoff[x][sub] : kOob, base);
        };
        v4i bq[2][2][BF];     // [set][sub][y]
        auto read_b = [&](int set, int buf, int t) {
            const int8_t* H = lds + (DB ? buf * halo_bytes : 0) + t_off[t];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int y = 0; y < BF; ++y)
                    bq[set][sub][y] = *reinterpret_cast<const v4i*>(H + bbyte[y] + 32 * sub);
        };
        fetch_halo(0);
#pragma unroll
        for (int t = 0; t < TAPS - 1; ++t) fetch_t(t, 0);
        stage_halo(0);
        __syncthreads();
        read_b(0, 0, 0);
        for (int kc = 0; kc < nkc; ++kc) {
            if (DB && kc + 1 < nkc) fetch_halo(kc + 1);
#pragma unroll
            for (int t = 0; t < TAPS; ++t) {
                // the tile of the step TAPS - 1 ahead: the previous tap's slot, of the next chunk unless t == 0
                fetch_t((t + TAPS - 1) % TAPS, t == 0 ? kc : kc + 1);
                if (t + 1 < TAPS) read_b((t + 1) & 1, kc & 1, t + 1);
#pragma unroll
                for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                    for (int x = 0; x < NX; ++x)
#pragma unroll
                        for (int y = 0; y < BF; ++y)
                            acc[x][y] = __builtin_amdgcn_mfma_i32_32x32x32_i8(rt[t][x][sub], bq[t & 1][sub][y], acc[x][y], 0, 0, 0);
            }
            if (DB && kc + 1 < nkc) {
                stage_halo((kc + 1) & 1);
                __syncthreads();
                read_b(0, (kc + 1) & 1, 0);
            }
        }
    } else {
        if (NS > 0) {
            fetch_halo(0);
    #pragma unroll
            for (int d = 0; d < kRingA - 1; ++d) fetch_a(d);
            stage_halo(0);
            __syncthreads();
        }

        // flat loop over steps (chunk outer, live tap inner), unrolled by the ring depth so that ring slots are constants
        int j = 0, kci = 0;
        for (int base = 0; base < NS; base += kRingA) {
    #pragma unroll
            for (int u = 0; u < kRingA; ++u) {
                if (base + u < NS) {   // uniform
                    fetch_a((u + kRingA - 1) % kRingA);                          // filter tiles of step s + kRingA - 1
                    if (DB && j == 0 && kci + 1 < nkc) fetch_halo(kci + 1);      // uniform; staged at the chunk's last tap
                    const int8_t* H = lds + (DB ? (kci & 1) * halo_bytes : 0) + 16 * lh;
                    const int ts = p.tap_slot[phase][j];
    #pragma unroll
                    for (int sub = 0; sub < 2; ++sub) {
                        v4i b[BF];
    #pragma unroll
                        for (int y = 0; y < BF; ++y)
                            b[y] = *reinterpret_cast<const v4i*>(H + (bslot[y] + ts) * kPitch + 32 * sub);
    #pragma unroll
                        for (int x = 0; x < NX; ++x)
    #pragma unroll
                            for (int y = 0; y < BF; ++y)
                                acc[x][y] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ra[u][x][sub], b[y], acc[x][y], 0, 0, 0);
                    }
                    if (j + 1 == taps) {
                        if (DB && kci + 1 < nkc) {
                            stage_halo((kci + 1) & 1);
                            __syncthreads();
                        }
                        j = 0;
                        ++kci;
                    } else {
                        ++j;
                    }
                }
            }
        }
    }

    // epilogue: register r of tile (x, y) is row 32x + 8*(r/4) + 4*lh + r%4, destination pixel q = wp*PXW + 32y + l32
    const int rowbase = row0 + wr * 64 + 4 * lh;
    const int HWd = p.Hd * p.Wd;
    const bool full_rows = row0 + ROWS <= p.Crow;
    if (ST == 2 && p.zfill && !p.bf16 && !p.acc_out && (p.Wd & 1) == 0) {   // uniform
        // Strided 1 x 1 layers, even rows: a pixel's 2 x 2 block leaves as (value, 0) and (0, 0), 8 bytes each.  The
        // result is four times the class image, so the lines a wave has touched but not yet completed outgrow the
        // L2 when its pixel fragments are written one after the other; here the fragments of one row (channel) are
        // written back to back instead, and the lines they share complete within a few instructions.
        float* o[BF];
        bool ok[BF], h1[BF];
#pragma unroll
        for (int y = 0; y < BF; ++y) {
            const int q = wp * PXW + 32 * y + l32;
            const int img = (int)fdiv((uint32_t)q, p.div_thw);
            const int rem = q - img * p.TH * p.TW;
            const int th = (int)fdiv((uint32_t)rem, p.div_tw);
            const int tw = rem - th * p.TW;
            const int n = n0 + img, h = (h0 + th) * ST, w = (w0 + tw) * ST;
            ok[y] = !(img >= p.NI || n >= p.N || h >= p.Hd || w >= p.Wd);
            h1[y] = h + 1 < p.Hd;
            o[y] = p.out + (((int64_t)n * p.Crow + rowbase) * HWd + h * p.Wd + w);
        }
#pragma unroll
        for (int x = 0; x < NX; ++x)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int dr = 32 * x + 8 * (r >> 2) + (r & 3);
                if (rowbase + dr >= p.Crow) continue;
#pragma unroll
                for (int y = 0; y < BF; ++y) {
                    if (!ok[y]) continue;
                    float* z = o[y] + (int64_t)dr * HWd;
                    *reinterpret_cast<float2*>(z) = make_float2((float)acc[x][y][r] * scale, 0.0f);
                    if (h1[y]) *reinterpret_cast<float2*>(z + p.Wd) = make_float2(0.0f, 0.0f);
                }
            }
        return;
    }
#pragma unroll
    for (int y = 0; y < BF; ++y) {
        const int q = wp * PXW + 32 * y + l32;
        const int img = (int)fdiv((uint32_t)q, p.div_thw);
        const int rem = q - img * p.TH * p.TW;
        const int th = (int)fdiv((uint32_t)rem, p.div_tw);
        const int tw = rem - th * p.TW;
        const int n = n0 + img, h = (h0 + th) * ST + pa, w = (w0 + tw) * ST + pb;
        if (img >= p.NI || n >= p.N || h >= p.Hd || w >= p.Wd) continue;
        const int64_t pix = ((int64_t)n * p.Crow + rowbase) * HWd + h * p.Wd + w;
        if (p.bf16) {   // uniform: the narrow result, same walk over the tile
            uint16_t* ob = reinterpret_cast<uint16_t*>(p.out) + pix;
            if (ST == 1 && (p.TW & 1) == 0 && (p.Wd & 1) == 0) {   // uniform
                // Even tile and image widths: lanes 2k and 2k+1 hold pixels w (even) and w+1 of one row, both inside the
                // image or both outside.  They trade values so that the even lane stores the pair of row dr and the odd
                // lane the pair of row dr+1, each as one aligned dword: half the store instructions, twice the bytes each.
                const bool odd = l32 & 1;
#pragma unroll
                for (int x = 0; x < NX; ++x)
#pragma unroll
                    for (int r = 0; r < 16; r += 2) {
                        const uint32_t v0 = bf16_bits((float)acc[x][y][r] * scale), v1 = bf16_bits((float)acc[x][y][r + 1] * scale);
                        const uint32_t got = (uint32_t)__builtin_amdgcn_mov_dpp((int)(odd ? v0 : v1), 0xB1, 0xF, 0xF, false);
                        const uint32_t word = odd ? (got | (v1 << 16)) : (v0 | (got << 16));
                        const int dr = 32 * x + 8 * (r >> 2) + (r & 3) + (odd ? 1 : 0);
                        if (rowbase + dr < p.Crow)
                            *reinterpret_cast<uint32_t*>(ob + (int64_t)dr * HWd - (odd ? 1 : 0)) = word;
                    }
                continue;
            }
            const bool w1 = w + 1 < p.Wd, h1 = h + 1 < p.Hd;
            const bool pairs = (p.Wd & 1) == 0;   // even rows: (value, 0) and (0, 0) go out as aligned 4-byte stores
#pragma unroll
            for (int x = 0; x < NX; ++x)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int dr = 32 * x + 8 * (r >> 2) + (r & 3);
                    if (rowbase + dr >= p.Crow) continue;
                    uint16_t* z = ob + (int64_t)dr * HWd;
                    const uint32_t v = bf16_bits((float)acc[x][y][r] * scale);
                    if (ST == 2 && p.zfill && pairs) {
                        *reinterpret_cast<uint32_t*>(z) = v;   // little endian: the value first, then the zero
                        if (h1) *reinterpret_cast<uint32_t*>(z + p.Wd) = 0u;
                    } else {
                        z[0] = (uint16_t)v;
                        if (ST == 2 && p.zfill) {
                            if (w1) z[1] = 0;
                            if (h1) z[p.Wd] = 0;
                            if (h1 && w1) z[p.Wd + 1] = 0;
                        }
                    }
                }
            continue;
        }
        float* o = p.out + pix;
        if (ST == 2 && p.zfill && (p.Wd & 1) == 0) {
            // written below together with the zeros of the 2 x 2 block
        } else if (full_rows && p.nt) {
#pragma unroll
            for (int x = 0; x < NX; ++x)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    __builtin_nontemporal_store((float)acc[x][y][r] * scale, &o[(32 * x + 8 * (r >> 2) + (r & 3)) * HWd]);
        } else if (full_rows) {
#pragma unroll
            for (int x = 0; x < NX; ++x)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[(32 * x + 8 * (r >> 2) + (r & 3)) * HWd] = (float)acc[x][y][r] * scale;
        } else {
#pragma unroll
            for (int x = 0; x < NX; ++x)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int dr = 32 * x + 8 * (r >> 2) + (r & 3);
                    if (rowbase + dr < p.Crow) o[dr * HWd] = (float)acc[x][y][r] * scale;
                }
        }
        if (p.acc_out) {
            int32_t* ao = p.acc_out + pix;
#pragma unroll
            for (int x = 0; x < NX; ++x)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int dr = 32 * x + 8 * (r >> 2) + (r & 3);
                    if (rowbase + dr < p.Crow) ao[dr * HWd] = acc[x][y][r];
                }
        }
        if (ST == 2 && p.zfill) {
            // the three neighbours of this pixel in its 2 x 2 block receive no tap at all
            const bool w1 = w + 1 < p.Wd, h1 = h + 1 < p.Hd;
            const bool pairs = (p.Wd & 1) == 0;   // even rows: (value, 0) and (0, 0) go out as aligned 8-byte stores
#pragma unroll
            for (int x = 0; x < NX; ++x)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int dr = 32 * x + 8 * (r >> 2) + (r & 3);
                    if (rowbase + dr >= p.Crow) continue;
                    float* z = o + (int64_t)dr * HWd;
                    if (pairs) {
                        *reinterpret_cast<float2*>(z) = make_float2((float)acc[x][y][r] * scale, 0.0f);
                        if (h1) *reinterpret_cast<float2*>(z + p.Wd) = make_float2(0.0f, 0.0f);
                    } else {
                        if (w1) z[1] = 0.0f;
                        if (h1) z[p.Wd] = 0.0f;
                        if (h1 && w1) z[p.Wd + 1] = 0.0f;
                    }
                    if (p.acc_out) {
                        int32_t* za = p.acc_out + pix + (int64_t)dr * HWd;
                        if (w1) za[1] = 0;
                        if (h1) za[p.Wd] = 0;
                        if (h1 && w1) za[p.Wd + 1] = 0;
                    }
                }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// 1 x 1 data gradient (and forward pass) at unit stride with a short contraction axis (at most 256 channels: for the
// data gradient the projection layers of MobileNetV2 and the 1 x 1 layers of ResNet-50 that reduce to 64 - 256 channels).  Such a layer is a few
// multiplies per 32 x 32 block of its result and is bound by that fp32 result; as a tile kernel (one to four steps
// per workgroup) it spent as long in set-up as in stores.  Here a wave streams: it keeps the filter fragments of
// two 32-row blocks of the result in registers (16 bytes per lane and 32-byte contraction step, from the
// fragment-order copy) and walks over groups of 32 consecutive pixels with a stride - the pixel fragments are 16
// bytes per lane straight from the NHWC gradient (coalesced, no LDS; the next group's are requested before the
// current group's multiplies), then 2 x KS v_mfma_i32_32x32x32_i8 and 32 stores of 128-byte runs per group.
// Waves of a workgroup hold neighbouring row blocks of the same pixel groups.
// ---------------------------------------------------------------------------------------------
struct StreamArgs {
    const int8_t* src;    // NHWC gradient, [pixels][cp]
    const int8_t* wfrag;  // filter in fragment order (one tap): [cp/64][RB][2][1024]
    uint32_t src_bytes, wfrag_bytes;
    int cp, Crow, RB, HW;
    int RP, S;            // pairs of row blocks; pixel-group phases, a multiple of four (a wave takes groups s, s + S, ...)
    uint32_t total_px, groups;
    FastDiv div_rp, div_hw;
    const float* s_a;
    const float* s_b;
    float* out;
    int32_t* acc_out;
    int nt;
    DwTail tail;          // tail.blocks > 0: that many workgroups behind the first main_blocks finish a deferred filter gradient
    int main_blocks;
    int bf16;             // the result is bfloat16 storage
};

// KS = 32-byte contraction steps (cp <= 32 * KS)
template <int KS>
__global__ __launch_bounds__(256) void k_dx_1x1_stream(StreamArgs p) {
    __shared__ int32_t l_role[256];
    if (p.tail.blocks > 0 && (int)blockIdx.x >= p.main_blocks) {   // uniform
        dw_reduce_role(p.tail, (int)blockIdx.x - p.main_blocks, l_role);
        return;
    }
    const int lane = threadIdx.x % kWave, l32 = lane & 31, lh = lane >> 5;
    // the four waves of a workgroup take four neighbouring pixel groups of one pair of row blocks: together they
    // write 512 consecutive bytes of each of the pair's 64 planes
    const uint32_t quad = fdiv(blockIdx.x, p.div_rp);
    const int rp = (int)(blockIdx.x - quad * (uint32_t)p.RP);
    const uint32_t s = quad * 4u + threadIdx.x / kWave;
    if (s >= (uint32_t)p.S) return;   // uniform per wave
    // (a wave takes groups s, s + S, ...: all waves together advance through the pixels as one window.  Giving every
    // workgroup a contiguous range of its own instead measured 13 % slower over ResNet-50's 17 such layers.)
    const __amdgpu_buffer_rsrc_t rs_src = __builtin_amdgcn_make_buffer_rsrc((void*)p.src, 0, (int)p.src_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc((void*)p.wfrag, 0, (int)p.wfrag_bytes, 0x00020000);
    const float scale = (*p.s_a / 127.0f) * (*p.s_b / 127.0f);

    v4i A[2][KS];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int rb = 2 * rp + j;
            const bool live = rb < p.RB && 32 * ks < p.cp;
            A[j][ks] = buffer_load16(rs_w, live ? (uint32_t)((((ks >> 1) * p.RB + rb) * 2 + (ks & 1)) * 1024 + lane * 16) : kOob, 0);
        }
    // contraction bytes 32*ks + 16*lh .. +15 of the lane's pixel; bytes past the channel pitch belong to the next pixel
    auto fetch = [&](uint32_t grp, v4i (&B)[KS]) {
        const uint32_t P = grp * 32u + (uint32_t)l32;
        const bool valid = grp < p.groups && P < p.total_px;
        const uint32_t boff = P * (uint32_t)p.cp + 16u * lh;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) B[ks] = buffer_load16(rs_src, (valid && 32 * ks + 16 * lh < p.cp) ? boff : kOob, 32u * ks);
    };
    v4i B[KS];
    fetch(s, B);
    for (uint32_t grp = s; grp < p.groups; grp += (uint32_t)p.S) {
        v4i Bn[KS];
        fetch(grp + (uint32_t)p.S, Bn);
        v16i acc[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][r] = 0;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[j][ks], B[ks], acc[j], 0, 0, 0);
        }
        const uint32_t P = grp * 32u + (uint32_t)l32;
        if (P < p.total_px) {
            const uint32_t n = fdiv(P, p.div_hw);
            const uint32_t r0 = P - n * (uint32_t)p.HW;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int rowbase = 32 * (2 * rp + j) + 4 * lh;
                const int64_t at = ((int64_t)n * p.Crow + rowbase) * p.HW + r0;
                if (p.bf16) {   // uniform
                    uint16_t* ob = reinterpret_cast<uint16_t*>(p.out) + at;
                    if ((p.HW & 1) == 0) {
                        // Even planes: lanes 2k and 2k+1 hold pixels r0 (even) and r0 + 1 of one plane.  They trade values so
                        // that the even lane stores the pair of row dr and the odd lane the pair of row dr + 1, each as one
                        // aligned dword: half the store instructions, twice the bytes each.
                        const bool odd = l32 & 1;
#pragma unroll
                        for (int r = 0; r < 16; r += 2) {
                            const uint32_t v0 = bf16_bits((float)acc[j][r] * scale), v1 = bf16_bits((float)acc[j][r + 1] * scale);
                            const uint32_t got = (uint32_t)__builtin_amdgcn_mov_dpp((int)(odd ? v0 : v1), 0xB1, 0xF, 0xF, false);
                            const uint32_t word = odd ? (got | (v1 << 16)) : (v0 | (got << 16));
                            const int dr = 8 * (r >> 2) + (r & 3) + (odd ? 1 : 0);
                            if (rowbase + dr < p.Crow) {
                                uint32_t* z = reinterpret_cast<uint32_t*>(ob + (int64_t)dr * p.HW - (odd ? 1 : 0));
                                if (p.nt) __builtin_nontemporal_store(word, z);
                                else *z = word;
                            }
                        }
                    } else {
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int dr = 8 * (r >> 2) + (r & 3);
                            if (rowbase + dr < p.Crow) ob[(int64_t)dr * p.HW] = (uint16_t)bf16_bits((float)acc[j][r] * scale);
                        }
                    }
                    continue;
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int dr = 8 * (r >> 2) + (r & 3);
                    if (rowbase + dr >= p.Crow) continue;
                    float* z = p.out + at + (int64_t)dr * p.HW;
                    if (p.nt) __builtin_nontemporal_store((float)acc[j][r] * scale, z);
                    else *z = (float)acc[j][r] * scale;
                    if (p.acc_out) p.acc_out[at + (int64_t)dr * p.HW] = acc[j][r];
                }
            }
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) B[ks] = Bn[ks];
    }
}

// Workgroups of one row tile: one per pixel tile, times the parity classes of a strided data gradient (whose tiles are
// padded to groups of eight, see the kernel's block decoding).
int64_t blocks_per_row_tile(const HaloArgs& a) {
    const int64_t per_phase = (int64_t)a.groups * a.tiles_h * a.tiles_w;
    if (a.stride > 1 && !a.zfill) return round_up(per_phase, 8) * a.stride * a.stride;
    return per_phase;
}

// floor division for possibly negative numerators
int floor_div(int a, int b) { return a >= 0 ? a / b : -((-a + b - 1) / b); }

struct Geometry {
    bool ok;
    HaloArgs a;
    size_t lds_bytes;
    int rows;
    int px;   // destination pixels per workgroup
};

// 1 x 1 filters with several contraction chunks, on 64-row tiles: the form with rings of chunks.  Unit stride, or
// stride 2 without padding (one live parity class whose workgroups also write the zeros of the other three: the
// contraction loop is the same, only the block decoding and the epilogue know about the stride).
bool ring1_applies(const Geometry& g) {
    const HaloArgs& a = g.a;
    return (a.stride == 1 || a.zfill) && a.T == 1 && a.ph_taps[0] == 1 && a.tap_slot[0][0] == 0 && a.double_buffer &&
           a.units <= g.px / 64 && g.rows == 64;
}

// backward: destination (h, w) of parity class (pa, pb), h = 2*th + pa, reads source row th + (pa + pad - kh*dil)/stride
// for every kh that makes the quotient exact.  forward (unit stride): source row = h - pad + kh*dil.
Geometry plan(bool backward, int N, int Hs, int Ws, int cp, int Hd, int Wd, int Crow, int kH, int kW, int sH, int sW,
              int pH, int pW, int dH, int dW, int px = kPxWg) {
    Geometry g{};
    g.px = px;
    HaloArgs& a = g.a;
    if (sH != sW || (sH != 1 && !(sH == 2 && backward)) || kH * kW > kMaxTaps) return g;
    // strided 1x1: three of four parity classes are empty; served when the live one is class (0, 0) (no padding),
    // whose workgroups then write the zeros of the other three next to their own results
    if (kH * kW == 1 && sH != 1 && (pH != 0 || pW != 0)) return g;
    a.zfill = (kH * kW == 1 && sH == 2) ? 1 : 0;
    const int s = sH;
    a.stride = s;
    a.T = kH * kW;
    int span_h = 0, span_w = 0;
    struct Tap { int oh, ow, id; };
    for (int ph = 0; ph < s * s; ++ph) {
        const int pa = ph / s, pb = ph % s;
        Tap taps[kMaxTaps];
        int nt = 0, mn_h = 1 << 30, mx_h = -(1 << 30), mn_w = 1 << 30, mx_w = -(1 << 30);
        for (int kh = 0; kh < kH; ++kh)
            for (int kw = 0; kw < kW; ++kw) {
                int oh, ow;
                if (backward) {
                    const int th = pa + pH - kh * dH, tw = pb + pW - kw * dW;
                    if (((th % s) + s) % s || ((tw % s) + s) % s) continue;
                    oh = floor_div(th, s);
                    ow = floor_div(tw, s);
                } else {
                    oh = kh * dH - pH;
                    ow = kw * dW - pW;
                }
                taps[nt++] = Tap{oh, ow, kh * kW + kw};
                mn_h = std::min(mn_h, oh); mx_h = std::max(mx_h, oh);
                mn_w = std::min(mn_w, ow); mx_w = std::max(mx_w, ow);
            }
        a.ph_taps[ph] = nt;
        a.ph_org_h[ph] = nt ? mn_h : 0;
        a.ph_org_w[ph] = nt ? mn_w : 0;
        if (nt) {
            span_h = std::max(span_h, mx_h - mn_h);
            span_w = std::max(span_w, mx_w - mn_w);
        }
        for (int t = 0; t < nt; ++t) {
            // slot offsets are filled in below, once the window width is known
            a.tap_slot[ph][t] = ((taps[t].oh - a.ph_org_h[ph]) << 8) | (taps[t].ow - a.ph_org_w[ph]);
            a.tap_id[ph][t] = taps[t].id;
        }
    }
    if (span_h > 255 || span_w > 255) return g;
    // tile of one parity class: best coverage of the class image by 256-pixel tiles whose window fits
    const int PH = (int)ceil_div(Hd, s), PW = (int)ceil_div(Wd, s);
    double best = 0.0;
    int bTH = 0, bTW = 0, bNI = 0;
    if (PH * PW <= px) {
        bTH = PH; bTW = PW; bNI = px / (PH * PW);
        if ((int64_t)bNI * (bTH + span_h) * (bTW + span_w) > 64 * kMaxUnits) bNI = (64 * kMaxUnits) / ((bTH + span_h) * (bTW + span_w));
        if (bNI < 1) return g;
    } else {
        // widest tile among the best covers: the result is stored in runs of TW pixels
        for (int tw = std::min(PW, 128); tw >= 4; --tw) {
            const int th = std::min(px / tw, PH);
            if (th < 1) continue;
            if ((int64_t)(th + span_h) * (tw + span_w) > 64 * kMaxUnits) continue;
            const double eff = (double)PH * PW / ((double)ceil_div(PH, th) * ceil_div(PW, tw) * px);
            if (eff > best + 0.02) { best = eff; bTH = th; bTW = tw; }
        }
        bNI = 1;
        if (bTH == 0) return g;
    }
    a.TH = bTH; a.TW = bTW; a.NI = bNI;
    a.SH = bTH + span_h; a.SW = bTW + span_w;
    for (int ph = 0; ph < s * s; ++ph)
        for (int t = 0; t < a.ph_taps[ph]; ++t) {
            const int v = a.tap_slot[ph][t];
            a.tap_slot[ph][t] = (v >> 8) * a.SW + (v & 255);
        }
    const int S = a.NI * a.SH * a.SW;
    a.units = (int)ceil_div(S, 64);   // for four waves; the eight-wave form of 128-row tiles halves it at launch
    if (a.units > kMaxUnits) return g;
    a.N = N; a.Hs = Hs; a.Ws = Ws; a.cp = cp; a.Hd = Hd; a.Wd = Wd; a.Crow = Crow;
    a.RB = (int)ceil_div(Crow, 32);
    a.tiles_h = (int)ceil_div(PH, a.TH);
    a.tiles_w = (int)ceil_div(PW, a.TW);
    a.groups = (int)ceil_div(N, a.NI);
    a.double_buffer = cp > kKc;
    g.lds_bytes = (size_t)(a.double_buffer ? 2 : 1) * S * kPitch;
    if (g.lds_bytes > 150 * 1024) return g;
    // 128-row tiles reuse each pixel fragment twice as often, but only pay off when they still fill the chip
    const int64_t blocks128 = (int64_t)a.groups * a.tiles_h * a.tiles_w * (a.zfill ? 1 : s * s) * ceil_div(Crow, 128);
    g.rows = (Crow > 64 && blocks128 >= 256 && px == kPxWg) ? 128 : 64;
    // 1 x 1 filters with several contraction chunks do hardly any arithmetic per chunk, so a workgroup is as fast as its
    // requests come back: the ring form (64-row tiles, chunks requested three ahead, two workgroups per CU) was
    // measured faster than 128-row tiles up to a thousand of those (ResNet-50's 128 -> 512 at 28 x 28 and 1024 -> 512
    // at 14 x 14, N = 64: 19.9 -> 18.2 and 29.7 -> 23.2 us), slower beyond (256 -> 512 at 56 x 56: 103 -> 120 us)
    if (g.rows == 128 && blocks128 <= 1024) {
        g.rows = 64;
        if (!ring1_applies(g)) g.rows = 128;
    }
    a.div_tw = make_fastdiv((uint32_t)a.TW);
    a.div_thw = make_fastdiv((uint32_t)(a.TH * a.TW));
    a.div_sw = make_fastdiv((uint32_t)a.SW);
    a.div_si = make_fastdiv((uint32_t)(a.SH * a.SW));
    a.div_tiles_w = make_fastdiv((uint32_t)a.tiles_w);
    a.div_tiles_hw = make_fastdiv((uint32_t)(a.tiles_h * a.tiles_w));
    const int64_t pt = blocks_per_row_tile(a);
    // room for the workgroups of a deferred filter-gradient reduction (at most 4096, dw_tail_worthwhile) is kept here,
    // so that the grid-size test of the launch cannot fail once an entry point has started launching
    if (pt * ceil_div(Crow, 64) >= ((int64_t)1 << 31) - 4096) return g;
    a.div_ptiles = make_fastdiv((uint32_t)pt);
    g.ok = true;
    return g;
}

// Profile labels, one per kernel form (they are different instantiations with different bounds): the tile kernel with
// a run-time tap list at unit stride, by parity classes at stride 2, on 128-row tiles, and the two constant-tap forms.
struct HaloNames { const char *dyn, *s2, *r128, *k1, *k9; };
constexpr HaloNames kBwdNames{"conv_bwd_data_halo", "conv_bwd_data_halo_s2", "conv_bwd_data_halo_r128", "conv_bwd_data_halo_1x1",
                              "conv_bwd_data_halo_3x3"};
constexpr HaloNames kFwdNames{"conv_fwd_halo", "conv_fwd_halo", "conv_fwd_halo_r128", "conv_fwd_halo_1x1", "conv_fwd_halo_3x3"};

// The ring form holds two workgroups per CU.  A layer whose 256-pixel tiles give far fewer than that (the late 1 x 1
// layers of a classification network: few pixels, long contraction) is cut into 128-pixel tiles instead.  Measured
// on ResNet-50's last stages, N = 64: 512 -> 2048 at 7 x 7 (104 tiles) 23.3 -> 17.2 us, 256 -> 1024 at 14 x 14 (256
// tiles) 14.6 -> 14.5 us cold and 12.4 -> 11.6 us warm, 2048 -> 512 at 7 x 7 (416 tiles) 14.0 -> 15.1 us: not there.
// The constant-tap 3 x 3 form (one workgroup per CU at 256 pixels) takes 128-pixel tiles below 192 tiles: 512 -> 512
// at 7 x 7, N = 64, has 104.
bool taps9_applies(const Geometry& g) {
    const HaloArgs& a = g.a;
    return a.stride == 1 && a.ph_taps[0] == 9 && a.double_buffer && g.rows == 64;
}

template <typename Plan>
Geometry plan_small(Geometry g, Plan replan) {
    if (!g.ok) return g;
    const int64_t blocks = blocks_per_row_tile(g.a) * ceil_div(g.a.Crow, 64);
    if (ring1_applies(g) && blocks < 384) {
        Geometry s = replan(128);
        return s.ok && ring1_applies(s) ? s : g;
    }
    if (taps9_applies(g) && blocks < 192) {
        Geometry s = replan(128);
        return s.ok && taps9_applies(s) ? s : g;
    }
    return g;
}

daq_status launch(Geometry& g, hipStream_t st, const HaloNames& names) {
    const HaloArgs& a = g.a;
    const char* name = g.rows == 128 ? names.r128 : a.stride == 2 ? names.s2 : names.dyn;
    const int64_t ptiles = blocks_per_row_tile(a);
    const int64_t blocks = ptiles * ceil_div(a.Crow, g.rows) + a.tail.blocks;
    if (blocks >= ((int64_t)1 << 31)) return DAQ_ERR_UNSUPPORTED;
    g.a.main_blocks = (int)(blocks - a.tail.blocks);
    if (a.tail.blocks > 0) g.lds_bytes = std::max<size_t>(g.lds_bytes, 8 * kWave * sizeof(int32_t));   // the role's scratch
    const dim3 grid((unsigned)blocks);
#define DAQ_HALO_CASE(WRV, DBV, WV)                                                                                  \
    {                                                                                                                \
        auto kern = a.stride == 2 ? k_conv_halo<WRV, DBV, 2, WV> : k_conv_halo<WRV, DBV, 1, WV>;                     \
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)g.lds_bytes) !=  \
            hipSuccess)                                                                                              \
            return DAQ_ERR_HIP;                                                                                      \
        DAQ_LAUNCH(name, st, hipLaunchKernelGGL(kern, grid, dim3(64 * WV), g.lds_bytes, st, a));                     \
    }
    // Layers with several contraction chunks and 3 x 3 filters at unit stride, on 64-row tiles: the form with a
    // constant tap count.  (With a single chunk the kernel is all prologue and epilogue, and the dynamic form, which
    // needs fewer registers, lets more workgroups overlap theirs; 128-row tiles stay on the eight-wave form.)
    // 1 x 1 filters with several contraction chunks, on 64-row tiles: the form with rings of chunks
    // (on 128-row tiles, which are chosen when the grid is large, it measured no better than the dynamic form)
    const bool ring1 = ring1_applies(g);
    if (g.px != kPxWg && !ring1 && !taps9_applies(g)) return DAQ_ERR_UNSUPPORTED;   // small tiles exist in these two forms only (see plan_small)
    if (ring1) {
        auto kern = a.stride == 2 ? (g.px == kPxWg ? k_conv_halo<1, true, 2, 4, 1> : k_conv_halo<1, true, 2, 4, 1, 2, 128>)
                                  : (g.px == kPxWg ? k_conv_halo<1, true, 1, 4, 1> : k_conv_halo<1, true, 1, 4, 1, 2, 128>);
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)g.lds_bytes) != hipSuccess)
            return DAQ_ERR_HIP;
        DAQ_LAUNCH(names.k1, st, hipLaunchKernelGGL(kern, grid, dim3(256), g.lds_bytes, st, a));
        return DAQ_OK;
    }
    if (taps9_applies(g)) {
        auto kern = g.px == kPxWg ? k_conv_halo<1, true, 1, 4, 9> : k_conv_halo<1, true, 1, 4, 9, 2, 128>;
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)g.lds_bytes) != hipSuccess)
            return DAQ_ERR_HIP;
        DAQ_LAUNCH(names.k9, st, hipLaunchKernelGGL(kern, grid, dim3(256), g.lds_bytes, st, a));
        return DAQ_OK;
    }
    if (g.rows == 128) {
        HaloArgs a8 = g.a;   // eight waves stage the window in half as many passes
        a8.units = (int)ceil_div((int64_t)g.a.NI * g.a.SH * g.a.SW, 128);
        const HaloArgs& a = a8;
        if (a.double_buffer) DAQ_HALO_CASE(2, true, 8) else DAQ_HALO_CASE(2, false, 8)
    } else if (a.Crow <= 32) {
#define DAQ_HALO_NARROW(DBV)                                                                                         \
    {                                                                                                                \
        auto kern = a.stride == 2 ? k_conv_halo<1, DBV, 2, 4, 0, 1> : k_conv_halo<1, DBV, 1, 4, 0, 1>;               \
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)g.lds_bytes) !=  \
            hipSuccess)                                                                                              \
            return DAQ_ERR_HIP;                                                                                      \
        DAQ_LAUNCH(name, st, hipLaunchKernelGGL(kern, grid, dim3(256), g.lds_bytes, st, a));                         \
    }
        if (a.double_buffer) DAQ_HALO_NARROW(true) else DAQ_HALO_NARROW(false)
#undef DAQ_HALO_NARROW
    } else {
        if (a.double_buffer) DAQ_HALO_CASE(1, true, 4) else DAQ_HALO_CASE(1, false, 4)
    }
#undef DAQ_HALO_CASE
    return DAQ_OK;
}

Geometry plan_bwd(const daq_conv_desc& d) {
    daq_layout Lg;
    daq_wpack_layout Lw;
    Geometry g{};
    if (d.groups != 1 || daq_layout_qg(&d, &Lg) != DAQ_OK || daq_layout_qw(&d, &Lw) != DAQ_OK) return g;
    if (Lg.kind != DAQ_LAYOUT_NHWC || Lg.bytes >= ((int64_t)1 << 31) || Lw.bytes - Lw.off_bwd_frag >= ((int64_t)1 << 31)) return g;
    auto make = [&](int px) {
        return plan(true, d.N, Lg.H, Lg.W, Lg.c_pitch, d.Hin, d.Win, d.Cin, d.kH, d.kW, d.strideH, d.strideW, d.padH, d.padW,
                    d.dilH, d.dilW, px);
    };
    g = plan_small(make(kPxWg), make);
    g.a.src_bytes = (uint32_t)Lg.bytes;
    g.a.wfrag_bytes = (uint32_t)(Lw.bytes - Lw.off_bwd_frag);
    return g;
}

Geometry plan_fwd(const daq_conv_desc& d) {
    daq_layout Lx;
    daq_wpack_layout Lw;
    Geometry g{};
    if (d.groups != 1 || daq_layout_qx_nhwc(&d, &Lx) != DAQ_OK || daq_layout_qw(&d, &Lw) != DAQ_OK) return g;
    if (Lx.bytes >= ((int64_t)1 << 31) || Lw.off_bwd_frag - Lw.off_fwd_frag >= ((int64_t)1 << 31)) return g;
    auto make = [&](int px) {
        return plan(false, d.N, d.Hin, d.Win, Lx.c_pitch, daq_out_h(&d), daq_out_w(&d), d.Cout, d.kH, d.kW, d.strideH,
                    d.strideW, d.padH, d.padW, d.dilH, d.dilW, px);
    };
    g = plan_small(make(kPxWg), make);
    g.a.src_bytes = (uint32_t)Lx.bytes;
    g.a.wfrag_bytes = (uint32_t)(Lw.off_bwd_frag - Lw.off_fwd_frag);
    return g;
}

// The streaming form serves: 1 x 1, unit stride, no padding, dense, at most 256 output channels.
bool stream_applies(const daq_conv_desc& d, const daq_layout& Lg) {
    return d.groups == 1 && d.kH == 1 && d.kW == 1 && d.strideH == 1 && d.strideW == 1 && d.padH == 0 && d.padW == 0 &&
           Lg.kind == DAQ_LAYOUT_NHWC && Lg.c_pitch <= 256 && (int64_t)d.N * d.Hin * d.Win < ((int64_t)1 << 31) - 64 &&
           ceil_div(std::max(d.Cin, d.Cout), 64) <= 4096;
}

// src: the NHWC operand (layout Ls); wfrag: the fragment-order filter copy whose rows are the result's `rows` channels
daq_status launch_stream(const char* name, const daq_conv_desc& d, const daq_layout& Ls, const int8_t* src,
                         const int8_t* wfrag, int64_t wfrag_bytes, int rows, const float* s_a, const float* s_b, float* out,
                         int32_t* acc, hipStream_t st, const DwTail* tail, bool bf16 = false) {
    StreamArgs a{};
    a.src = src;
    a.wfrag = wfrag;
    a.src_bytes = (uint32_t)Ls.bytes;
    a.wfrag_bytes = (uint32_t)wfrag_bytes;
    a.cp = Ls.c_pitch;
    a.Crow = rows;
    a.RB = (int)ceil_div(rows, 32);
    a.HW = d.Hin * d.Win;
    a.total_px = (uint32_t)((int64_t)d.N * a.HW);
    a.groups = (uint32_t)ceil_div((int64_t)a.total_px, 32);
    a.RP = (int)ceil_div(a.RB, 2);
    const int ks = (int)ceil_div(a.cp, 32);
    // waves the chip holds at this form's register count; a wave should get several groups for its filter fragments
    const int64_t target = ks <= 2 ? 8192 : ks <= 4 ? 4096 : 2048;
    a.S = (int)round_up(std::max<int64_t>(1, std::min<int64_t>(ceil_div((int64_t)a.groups, 2), target / a.RP)), 4);
    a.div_rp = make_fastdiv((uint32_t)a.RP);
    a.div_hw = make_fastdiv((uint32_t)a.HW);
    a.s_a = s_a; a.s_b = s_b;
    a.out = out; a.acc_out = acc;
    a.bf16 = bf16 ? 1 : 0;
    a.nt = (int64_t)d.N * rows * a.HW * (bf16 ? 2 : 4) >= kStreamBytes;
    const int64_t wgs = (int64_t)a.RP * ceil_div(a.S, 4);
    if (tail) a.tail = *tail;
    a.main_blocks = (int)wgs;
    const dim3 grid((unsigned)(wgs + a.tail.blocks));
#define DAQ_STREAM(KSV) DAQ_LAUNCH(name, st, hipLaunchKernelGGL((k_dx_1x1_stream<KSV>), grid, dim3(256), 0, st, a))
    if (ks <= 1) DAQ_STREAM(1);
    else if (ks <= 2) DAQ_STREAM(2);
    else if (ks <= 4) DAQ_STREAM(4);
    else DAQ_STREAM(8);
#undef DAQ_STREAM
    return DAQ_OK;
}

}  // namespace

bool bwd_data_halo_supported(const daq_conv_desc& d) { return plan_bwd(d).ok; }

daq_status conv_bwd_data_halo(const daq_conv_desc& d, const int8_t* qg, const float* s_g, const int8_t* qw,
                              const float* s_w, float* dX, int32_t* acc, hipStream_t st, const DwTail* tail, bool bf16) {
    Geometry g = plan_bwd(d);
    if (tail) g.a.tail = *tail;
    g.a.bf16 = bf16 ? 1 : 0;
    daq_wpack_layout Lw;
    if (!g.ok || daq_layout_qw(&d, &Lw) != DAQ_OK) return DAQ_ERR_UNSUPPORTED;
    daq_layout Lg;
    if (daq_layout_qg(&d, &Lg) == DAQ_OK && stream_applies(d, Lg))
        return launch_stream("conv_bwd_data_stream", d, Lg, qg, qw + Lw.off_bwd_frag, Lw.bytes - Lw.off_bwd_frag, d.Cin, s_w, s_g, dX, acc,
                             st, tail, bf16);
    g.a.src = qg;
    g.a.wfrag = qw + Lw.off_bwd_frag;
    g.a.s_a = s_w; g.a.s_b = s_g;
    g.a.out = dX; g.a.acc_out = acc;
    g.a.nt = !bf16 && (int64_t)d.N * d.Cin * d.Hin * d.Win * 4 >= kStreamBytes;
    return launch(g, st, kBwdNames);
}

bool fwd_halo_supported(const daq_conv_desc& d) { return plan_fwd(d).ok; }

daq_status conv_fwd_halo(const daq_conv_desc& d, const int8_t* qx, const int8_t* qw, const float* s_x, const float* s_w,
                         float* Y, int32_t* acc, hipStream_t st) {
    Geometry g = plan_fwd(d);
    daq_wpack_layout Lw;
    if (!g.ok || daq_layout_qw(&d, &Lw) != DAQ_OK) return DAQ_ERR_UNSUPPORTED;
    daq_layout Lx;
    if (daq_layout_qx_nhwc(&d, &Lx) == DAQ_OK && stream_applies(d, Lx))   // thin 1 x 1 layers: the streaming kernel, rows = Cout
        return launch_stream("conv_fwd_stream", d, Lx, qx, qw + Lw.off_fwd_frag, Lw.off_bwd_frag - Lw.off_fwd_frag, d.Cout, s_x, s_w, Y,
                             acc, st, nullptr);
    g.a.src = qx;
    g.a.wfrag = qw + Lw.off_fwd_frag;
    g.a.s_a = s_x; g.a.s_b = s_w;
    g.a.out = Y; g.a.acc_out = acc;
    g.a.nt = (int64_t)d.N * d.Cout * daq_out_h(&d) * daq_out_w(&d) * 4 >= kStreamBytes;
    return launch(g, st, kFwdNames);
}

}  // namespace daq
