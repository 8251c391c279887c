// Gradient Vectorized Quantization on gfx950: channel statistics, discriminator + clip solve,
// and the int8 packing kernels (Algorithm 1, per-channel loop and the two quantizations), plus
// the per-tensor quantization of X and W used by the forward pass.
//
// All kernels here are meant to be bandwidth bound, which on this chip takes care with the instruction count too
// (buffer loads instead of selects, 24-bit multiplies, one-instruction rounding).  Float reductions use fixed
// trees and a fixed-order second stage (no float atomics), so results do not depend on scheduling.  Compile with
// -ffp-contract=off: the rounding of every fp32/fp64 expression below is part of the contract.
#include <algorithm>
#include <cmath>
#include <mutex>

#include "daq_internal.h"

namespace daq {

namespace {

typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef uint32_t v2u __attribute__((ext_vector_type(2)));

constexpr int kBlock = 256;
constexpr int kStatsElems = 4096;  // elements one statistics workgroup sweeps per iteration (16 per thread, all in flight)
constexpr int kMaxSlabs = 16;      // statistics partials per channel (every consumer re-folds them)
constexpr int kCountGrid = 1024;   // workgroups the counting pass aims for; one count partial per channel each
constexpr int64_t kEarlyVqMinElems = (int64_t)8 << 20;   // gradients from this size on take the early per-channel copy

// ---------------------------------------------------------------------------------------------
// workspace carving
// ---------------------------------------------------------------------------------------------
struct QuantWs {
    float* gmax;          // [C]  |g|max, mean, sigma: written by the counting pass for the packing pass
    float* mean;          // [C]
    float* sigma;         // [C]
    float* s_prev;        // [C]  copy of the clip state taken before anything overwrites it
    uint32_t* pred;       // [C]  class the counting pass assumed when it wrote the per-channel copy early (see k_count_qg)
    float* layer;         // [8]  whole-tensor values for the ablation schemes: |g|max (not zeroed when tiny), mean, sigma,
                          //      tail mass P, clip value, class
    uint32_t* layer_cnt;  // [counting waves]  #{|g| > sigma} over all 16 channels of a counting wave (layer-wise clipping)
    float* part_max;      // [C][slabs]
    double* part_s1;      // [C][slabs]
    double* part_s2;      // [C][slabs]
    uint32_t* part_cnt;   // [C][cgroups]  #{|g| > sigma} seen by counting workgroup p of the channel's block
    int chunks;           // 4096-element chunks of one channel
    int slabs;            // statistics workgroups (partials) per channel
    int tiles;            // 64-pixel tiles of the flattened (n, h*w) axis
    int cgroups;          // counting workgroups per block of 64 channels
    int scheme;           // daq_scheme the launches of this call follow
    int64_t total_bytes;
};

QuantWs carve_quant_ws(void* base, int C, int N, int HW) {
    QuantWs w{};
    const int64_t M = (int64_t)N * HW;
    // statistics sweep groups of four elements per plane (k_stats): the axis is padded to whole groups
    const int64_t Mstats = HW >= 4 ? (int64_t)N * ((HW + 3) / 4) * 4 : M;
    w.chunks = (int)ceil_div(Mstats, kStatsElems);
    const int iters = (int)ceil_div(w.chunks, kMaxSlabs);
    w.slabs = (int)ceil_div(w.chunks, iters);
    w.tiles = (int)ceil_div(M, kWave);
    const int cb = (int)ceil_div(C, 64);
    const int want = std::max(1, kCountGrid / cb);
    const int titers = (int)ceil_div(w.tiles, want);
    w.cgroups = (int)ceil_div(w.tiles, titers);
    if (w.cgroups >= 2 * kXcd) w.cgroups = (int)round_up(w.cgroups, kXcd);   // whole rounds over the XCDs (see k_count_qg)
    // byte offsets first; pointers only when there is a buffer (a size query passes none)
    int64_t off = 0;
    const int64_t o_head = off;
    off += round_up(((int64_t)5 * C + 8) * 4, 256);
    const int64_t o_s1 = off;
    off += round_up((int64_t)2 * C * w.slabs * 8, 256);
    const int64_t o_max = off;
    off += round_up((int64_t)C * w.slabs * 4, 256);
    const int64_t o_cnt = off;
    off += round_up((int64_t)C * w.cgroups * 4, 256);
    const int64_t o_lcnt = off;
    off += round_up((int64_t)cb * w.cgroups * (kBlock / kWave) * 4, 256);
    w.total_bytes = off;
    if (base) {
        char* p = (char*)base;
        w.gmax = (float*)(p + o_head);
        w.mean = w.gmax + C;
        w.sigma = w.mean + C;
        w.s_prev = w.sigma + C;
        w.pred = (uint32_t*)(w.s_prev + C);
        w.layer = (float*)(w.pred + C);
        w.part_s1 = (double*)(p + o_s1);
        w.part_s2 = w.part_s1 + (int64_t)C * w.slabs;
        w.part_max = (float*)(p + o_max);
        w.part_cnt = (uint32_t*)(p + o_cnt);
        w.layer_cnt = (uint32_t*)(p + o_lcnt);
    }
    return w;
}

// ---------------------------------------------------------------------------------------------
// device helpers
// ---------------------------------------------------------------------------------------------
// Stochastic rounding: a counter-based generator on 32-bit arithmetic.  fmix32 is the finalizer of MurmurHash3
// (Appleby, public domain), a bijection of 32-bit words with full avalanche.  A launch derives one key from the
// caller's 64-bit seed (round_key, on the host); element i (its NCHW index, below 2^31) hashes once,
//     h = fmix32(i ^ key),
// and the two int8 copies take disjoint halves of the word as 16-bit uniforms: the per-channel copy (t = 0) U = h >> 16,
// the per-tensor copy (t = 1) U = h & 0xFFFF, u = U * 2^-16.  A kernel that writes both copies of an element pays for
// one hash (the calls below are pure, the compiler merges them); nothing is carried from one element to the next.
__host__ __device__ __forceinline__ uint32_t fmix32(uint32_t h) {
    h ^= h >> 16;
    h *= 0x85EBCA6Bu;
    h ^= h >> 13;
    h *= 0xC2B2AE35u;
    h ^= h >> 16;
    return h;
}
// key = fmix32(seed_lo ^ fmix32(seed_hi ^ 0x9E3779B9)); it travels in the kernels' 64-bit seed argument
inline uint64_t round_keys(uint64_t seed) {
    const uint32_t lo = (uint32_t)seed, hi = (uint32_t)(seed >> 32);
    return (uint64_t)fmix32(lo ^ fmix32(hi ^ 0x9E3779B9u));
}
__device__ __forceinline__ uint32_t rng_u(uint64_t keys, uint32_t tensor, uint32_t idx) {
    const uint32_t h = fmix32(idx ^ (uint32_t)keys);
    return tensor == 0u ? h >> 16 : h & 0xFFFFu;
}

// 127/s, or 0 when the scale is treated as zero (then every code is 0).
__device__ __forceinline__ float inv_scale(float s) { return (s >= kTinyScale) ? 127.0f / s : 0.0f; }

// Eq. "suq" in code space: round(clamp(x*inv, -127, 127)).  Stochastic rounding: floor(t) + [frac(t) > U * 2^-16] with
// the element's 16-bit draw U, evaluated in integers: with c = ceil(t * 2^16) (exact: |t| <= 127) the bracket is
// [c mod 2^16 > U] - a fraction of exactly 0 never rounds up, one above U * 2^-16 always - so the code is
// (c + 65535 - U) >> 16 with an arithmetic shift.
template <bool STOCH>
__device__ __forceinline__ int quant_code(float x, float inv, uint32_t U) {
    float t = x * inv;
    t = fminf(fmaxf(t, -127.0f), 127.0f);
    if (STOCH) {
        // -ceil(t * 2^16) = floor(-t * 2^16), floor and conversion in one instruction (|t * 2^16| < 2^23: exact)
        int nc;
        asm("v_cvt_flr_i32_f32 %0, %1" : "=v"(nc) : "v"(t * -65536.0f));
        return (65535 - (int)U - nc) >> 16;
    }
    return (int)rintf(t);
}

// The same code as quant_code, left in the low byte of a 32-bit word (upper bytes are don't-care).
// Nearest: adding 1.5 * 2^23 to a value of magnitude <= 127 rounds it to an integer, ties to even,
// and leaves that integer in two's complement in the low mantissa bits - one instruction instead of
// round + convert + mask.
template <bool STOCH>
__device__ __forceinline__ uint32_t quant_bits(float x, float inv, uint32_t U) {
    if (STOCH) return (uint32_t)quant_code<true>(x, inv, U);
    const float t = __builtin_amdgcn_fmed3f(x * inv, -127.0f, 127.0f);
    return __float_as_uint(t + 12582912.0f);
}
// Low bytes of four words -> one dword (a in byte 0).
__device__ __forceinline__ uint32_t pack4(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    const uint32_t lo = __builtin_amdgcn_perm(b, a, 0x0c0c0400u);
    const uint32_t hi = __builtin_amdgcn_perm(d, c, 0x0c0c0400u);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}

// fp32 tensors are read through a buffer descriptor with 32-bit byte offsets: an offset of kOobOff (or
// anything past the extent) returns 0.0f, which is how ragged tiles and padding positions are read
// without branches or selects on the loaded value.  Tensors must be smaller than 2 GiB.
constexpr uint32_t kOobOff = 0x80000000u;
__device__ __forceinline__ __amdgpu_buffer_rsrc_t f32_rsrc(const void* p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc((void*)p, 0, (int)bytes, 0x00020000);
}
// The tensor to quantize is fp32 (T = float) or bfloat16 (T = uint16_t, the upper half of the fp32 pattern: widening
// is exact, so everything downstream is the fp32 arithmetic on the widened values).  Offsets are in bytes of T.
__device__ __forceinline__ float widen_bf16(uint32_t b) { return __uint_as_float(b << 16); }
template <typename T>
__device__ __forceinline__ float buf_ld(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
    if constexpr (sizeof(T) == 4) return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, 0));
    else return widen_bf16((uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(r, (int)voff, (int)soff, 0));
}
// four consecutive elements as fp32 bit patterns / one element, or zeros (see ld16_or_zero)
template <typename T>
__device__ __forceinline__ uint4 ld4_or_zero(const T* p, bool ok) {
    if constexpr (sizeof(T) == 4) {
        return ld16_or_zero(p, ok);
    } else {
        typedef uint32_t u2_a2 __attribute__((ext_vector_type(2), aligned(2)));
        const u2_a2 v = *reinterpret_cast<const u2_a2*>(ok ? (const void*)p : (const void*)g_zero64);
        return make_uint4(v[0] << 16, v[0] & 0xffff0000u, v[1] << 16, v[1] & 0xffff0000u);
    }
}
template <typename T>
__device__ __forceinline__ float ld1_or_zero(const T* p, bool ok) {
    if constexpr (sizeof(T) == 4) return ldf_or_zero(p, ok);
    else return widen_bf16(*(ok ? p : reinterpret_cast<const uint16_t*>(g_zero64)));
}
__device__ __forceinline__ float buf_ldf(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
    return __uint_as_float((uint32_t)__builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, 0));
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_down(v, o));
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o);
    return v;
}
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o);
    return v;
}

__global__ void k_fill_u32(uint32_t* p, int64_t n, uint32_t v) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// Fixed-shape workgroup reduction of (max, sum, sum); the result is valid in thread 0.
__device__ __forceinline__ void block_reduce(float& mx, double& s1, double& s2) {
    __shared__ float l_mx[kBlock / kWave];
    __shared__ double l_s1[kBlock / kWave], l_s2[kBlock / kWave];
    mx = wave_max(mx);
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    if (lane == 0) { l_mx[wave] = mx; l_s1[wave] = s1; l_s2[wave] = s2; }
    __syncthreads();
    if (threadIdx.x == 0)
        for (int w = 1; w < kBlock / kWave; ++w) { mx = fmaxf(mx, l_mx[w]); s1 += l_s1[w]; s2 += l_s2[w]; }
}

// ---------------------------------------------------------------------------------------------
// S1: per-channel |g|max, sum, sum of squares.  Workgroup (c, j) sweeps the 4096-element chunks
// j, j + slabs, ... of channel c's flattened (n, h*w) axis, the loads of the next chunk in flight
// while the current one is reduced, and stores one partial.  A channel has at most 16 partials, so
// the kernels that need mean and sigma fold them again themselves (fold_stats) in a fixed order
// instead of waiting for a reduction launch.  Channel c runs on XCD c % 8 in every pass over dY.
// ---------------------------------------------------------------------------------------------
// TAIL: the plane size is not a multiple of four (the last group of a plane needs the move-back and the mask).
template <typename T, bool VEC4, bool TAIL>
__global__ __launch_bounds__(kBlock) void k_stats(const T* __restrict__ g, int N, int C, int HW, FastDiv div_hw,
                                                  QuantWs ws) {
    constexpr int NV = VEC4 ? 4 : 16;
    const int b = blockIdx.x;
    const int xcd = b % kXcd, q = b / kXcd;
    const int c = (q / ws.slabs) * kXcd + xcd;
    const int j = q % ws.slabs;
    if (c >= C) return;
    const int M = N * HW;
    const int tid = threadIdx.x;

    // VEC4: a thread takes groups of four consecutive elements of one (image, channel) plane, any plane size >= 4:
    // planes are cut into ceil(HW/4) groups and the last group of a plane is moved back to end with the plane (its
    // leading elements, already covered by the group before, are zeroed), so every load is a dword-aligned 16-byte
    // load inside the plane.  The flattened axis of a channel is then N * ceil(HW/4) * 4 element slots long.
    const int G4 = (HW + 3) >> 2;
    uint4 v[NV];   // VEC4: four floats each; otherwise only .x is used
    auto fetch = [&](int chunk, uint4 (&dst)[NV]) {
        const bool live = chunk < ws.chunks;
        const int m0 = chunk * kStatsElems;
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            if (VEC4) {
                const int q4 = (m0 >> 2) + tid + u * kBlock;            // group index inside the channel
                const bool ok = live && q4 < N * G4;
                const int qc = ok ? q4 : 0;
                const int n = (int)fdiv((uint32_t)qc, div_hw), gi = qc - n * G4;   // div_hw divides by G4 here
                const int i = TAIL ? min(4 * gi, HW - 4) : 4 * gi;
                uint4 r = ld4_or_zero<T>(g + ((int64_t)n * C + c) * HW + i, ok);
                if (TAIL) {
                    const int skip = 4 * gi - i;   // > 0 only in a plane's last group
                    r.x = skip > 0 ? 0u : r.x;
                    r.y = skip > 1 ? 0u : r.y;
                    r.z = skip > 2 ? 0u : r.z;
                }
                dst[u] = r;
            } else {
                const int m = m0 + tid + u * kBlock;
                const bool ok = live && m < M;
                const int mc = ok ? m : 0;
                const int n = (int)fdiv((uint32_t)mc, div_hw), i = mc - n * HW;
                dst[u].x = __float_as_uint(ld1_or_zero<T>(g + ((int64_t)n * C + c) * HW + i, ok));
            }
        }
    };
    float mx = 0.0f;
    double s1 = 0.0, s2 = 0.0;
    fetch(j, v);
    for (int chunk = j; chunk < ws.chunks; chunk += ws.slabs) {
        uint4 nv[NV];
        fetch(chunk + ws.slabs, nv);
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const float f0 = __uint_as_float(v[u].x);
            mx = fmaxf(mx, fabsf(f0));
            const double a = f0;
            s1 += a;
            s2 += a * a;
            if (VEC4) {
                const float f1 = __uint_as_float(v[u].y), f2 = __uint_as_float(v[u].z), f3 = __uint_as_float(v[u].w);
                mx = fmaxf(mx, fmaxf(fabsf(f1), fmaxf(fabsf(f2), fabsf(f3))));
                const double bq = f1, cq = f2, d = f3;
                s1 += bq; s1 += cq; s1 += d;
                s2 += bq * bq; s2 += cq * cq; s2 += d * d;
            }
        }
#pragma unroll
        for (int u = 0; u < NV; ++u) v[u] = nv[u];
    }
    block_reduce(mx, s1, s2);
    if (tid == 0) {
        const int64_t slot = (int64_t)c * ws.slabs + j;
        ws.part_max[slot] = mx;
        ws.part_s1[slot] = s1;
        ws.part_s2[slot] = s2;
    }
}

// Partials of channel c -> |g|max, mean, sigma (population std about the mean, fp64, rounded once).
// Sequential in slab order, so every workgroup that calls it gets the same bits.
__device__ __forceinline__ void fold_stats(const QuantWs& ws, int c, double Md, float& gmax, float& mean, float& sigma) {
    // all partials are requested before the first one is used; slots past `slabs` read zeros, which change nothing
    float pm[kMaxSlabs];
    double p1[kMaxSlabs], p2[kMaxSlabs];
#pragma unroll
    for (int j = 0; j < kMaxSlabs; ++j) {
        const bool ok = j < ws.slabs;
        const int64_t slot = (int64_t)c * ws.slabs + j;
        pm[j] = ldf_or_zero(ws.part_max + slot, ok);
        p1[j] = *(ok ? ws.part_s1 + slot : reinterpret_cast<const double*>(g_zero64));
        p2[j] = *(ok ? ws.part_s2 + slot : reinterpret_cast<const double*>(g_zero64));
    }
    float mx = 0.0f;
    double s1 = 0.0, s2 = 0.0;
#pragma unroll
    for (int j = 0; j < kMaxSlabs; ++j) {
        mx = fmaxf(mx, pm[j]);
        s1 += p1[j];
        s2 += p2[j];
    }
    const double mu = s1 / Md;
    double var = s2 / Md - mu * mu;
    if (var < 0.0) var = 0.0;
    gmax = mx;
    mean = (float)mu;
    sigma = (float)sqrt(var);
}

// S4: clip value of a channel of the given class (Eq. "gaus": |g|max; Eq. "fats": (1-kA) s_prev + A |g|max, with a
// non-positive state meaning "no history" and a non-positive result replaced by |g|max).
__device__ __forceinline__ float clip_rule(int klass, float gm, float prev, float k, float A) {
    float s = gm;
    if (klass == DAQ_CLASS_INVT) {
        if (!(prev > 0.0f)) prev = gm;
        s = (float)((1.0 - (double)k * (double)A) * (double)prev + (double)A * (double)gm);
        if (!(s > 0.0f)) s = gm;
    }
    return s;
}

// What the counting pass needs to write the per-channel copy of channels whose class it can guess.
struct EarlyVq {
    int8_t* vq;            // nullptr: the counting pass does not write the per-channel copy
    int64_t chan_pitch;
    int32_t lead, img_rows, row_pitch, W;
    FastDiv div_w;
    float k, A;
    float ratio;           // a channel with |g|max > ratio * sigma is taken for long-tailed
    int quad;              // rows are a multiple of four pixels long: four adjacent lanes hold four pixels of one row
};

// Value of `v` in the lane whose number differs in bit 0 (XOR1) or bit 1 (otherwise), by DPP quad permutation.
template <bool XOR1>
__device__ __forceinline__ uint32_t quad_swap(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, XOR1 ? 0xB1 : 0x4E, 0xF, 0xF, false);
}

// ---------------------------------------------------------------------------------------------
// S2 (+ the global copy of S5): tail-mass count per channel, fused with the globally quantized
// NHWC copy.  A workgroup owns 64 channels and walks 64-pixel tiles p, p + cgroups, ... of the
// flattened (n, h*w) axis; wave w handles channels 16w..16w+15 with lane = pixel, so every load is
// a 256-byte run of one channel and the lane's 16 codes are 16 contiguous bytes of the NHWC output.
// The workgroup first folds the statistics partials of its 64 channels (sigma) and of all channels
// (the global scale max_c |g|max), then counts with wave ballots into registers and stores one
// count partial per channel: no atomics, no reduction launch.
// ---------------------------------------------------------------------------------------------
//
// EARLY: the pass also writes the per-channel copy vq.  The class of a channel is only known once the counts of all
// its workgroups are in, but |g|max / sigma, known here, separates bell-shaped from long-tailed channels almost
// always: every workgroup derives the same guess and the clip value that follows from it (same arithmetic as the
// final decision), quantizes with it and stores the bytes of the real elements; the packing pass, which takes the
// decision, then only rewrites the channels whose guess was wrong (and writes the padding).  A correct guess saves
// the third sweep over dY for that channel; a wrong one costs nothing but the bytes written here.
template <typename T, bool STOCH, bool WRITE_QG, bool COUNT, bool EARLY = false>
__global__ __launch_bounds__(kBlock, 4) void k_count_qg(const T* __restrict__ g, int N, int C, int HW, int c_pitch,
                                                     FastDiv div_hw, QuantWs ws, const float* __restrict__ scale_ptr,
                                                     int8_t* __restrict__ qg, uint64_t seed,
                                                     const float* __restrict__ s_state, float* __restrict__ s_global,
                                                     EarlyVq ev, int qg_tail) {
    __shared__ float l_sigma[64];
    __shared__ float l_inv[64];
    __shared__ float l_max[kBlock / kWave];
    __shared__ __align__(16) int8_t l_tile[64 * 80];
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int p = blockIdx.x % ws.cgroups;
    const int cb = blockIdx.x / ws.cgroups;
    // A last block of at most 32 channels (thin tensors; channel counts like 96 or 144) has one or two groups of 16 channels,
    // and two or three of the four waves would idle.  Its waves take four (or two) different pixel tiles instead, and
    // since the block's share of an NHWC record is then 16 (or 32) bytes, a lane's codes are that share (or half of it):
    // stored directly, no transposition through LDS, no barrier in the loop.
    const int left = C - cb * 64;
    const int narrow = left <= 16 ? 1 : left <= 32 ? 2 : 0;   // uniform: groups of 16 channels
    const int sub = narrow ? wave / narrow : 0, nsub = narrow ? 4 / narrow : 1;   // the wave's pixel tile among the workgroup's
    const int c0 = cb * 64 + 16 * (narrow ? wave % narrow : wave);
    const int wg_tiles = (ws.tiles + nsub - 1) / nsub;
    const uint32_t M = (uint32_t)N * (uint32_t)HW;
    constexpr uint32_t EB = sizeof(T);   // bytes of a source element
    const __amdgpu_buffer_rsrc_t rs = f32_rsrc(g, (uint32_t)M * (uint32_t)C * EB);
    const uint32_t chan_bytes = (uint32_t)HW * EB;
    // (measured: a gain where the kernel only counts or writes one copy, a loss in the form that writes both copies)
    const bool dword16 = EB == 2 && !EARLY && (HW & 1) == 0 && ((uintptr_t)g & 3u) == 0;

    // Which tiles the workgroup walks.  A tile's 256-byte pieces of its channel planes start wherever the plane starts, so
    // neighbouring tiles share cache lines; with the workgroups of a channel block dealt round-robin over the tiles,
    // neighbours ran on different XCDs and both L2s fetched the shared lines (1.4 x the tensor on 14 x 14 planes).  With
    // a multiple of eight workgroups per block, workgroup p runs on XCD p % 8: each XCD takes one contiguous eighth of
    // the tiles, and its workgroups p / 8 walk that range side by side.
    int t_first = p, t_step = ws.cgroups, t_end = wg_tiles;
    if ((ws.cgroups & (kXcd - 1)) == 0) {   // uniform
        const int per_xcd = (wg_tiles + kXcd - 1) / kXcd, xcd = p % kXcd;
        t_first = xcd * per_xcd + p / kXcd;
        t_step = ws.cgroups / kXcd;
        t_end = min(wg_tiles, (xcd + 1) * per_xcd);
    }

    float x[16];
    uint32_t n_cur = 0, px_cur = 0;
    bool v_cur = false;
    auto fetch = [&](int tile, float (&dst)[16], uint32_t& n, uint32_t& px, bool& valid) {
        const uint32_t P = (uint32_t)(nsub * tile + sub) * kWave + lane;
        valid = tile < t_end && P < M;
        const uint32_t Pc = valid ? P : 0u;
        n = fdiv(Pc, div_hw);
        px = Pc - n * (uint32_t)HW;
        const uint32_t off = valid ? ((n * (uint32_t)C + (uint32_t)c0) * (uint32_t)HW + px) * EB : kOobOff;
        if (EB == 2 && dword16) {   // uniform
            // bfloat16 through dword loads (two-byte loads run at a fraction of the rate): the lane fetches the aligned
            // dword that holds its element - its neighbour fetches the same one - and keeps one half.  Planes start on
            // dword boundaries here (even plane size, aligned tensor), so the half is the same for all 16 channels.
            const uint32_t offa = valid ? (off & ~3u) : kOobOff;
            const bool upper = (off & 2u) != 0;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const uint32_t raw = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rs, (int)((c0 + i < C) ? offa : kOobOff), (int)((uint32_t)i * chan_bytes), 0);
                dst[i] = __uint_as_float(upper ? (raw & 0xffff0000u) : (raw << 16));
            }
        } else if (c0 + 16 <= C) {   // uniform per wave
#pragma unroll
            for (int i = 0; i < 16; ++i) dst[i] = buf_ld<T>(rs, off, (uint32_t)i * chan_bytes);
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) dst[i] = buf_ld<T>(rs, c0 + i < C ? off : kOobOff, (uint32_t)i * chan_bytes);
        }
    };
    fetch(t_first, x, n_cur, px_cur, v_cur);

    // scale of the global copy: max_c |g|max from the statistics pass, or an explicit per-tensor scale
    float sg = 0.0f;
    if (scale_ptr) {
        sg = *scale_ptr;
    } else {
        float m = 0.0f;
        const int total = C * ws.slabs;
        for (int base = 0; base < total; base += 8 * kBlock) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = ldf_or_zero(ws.part_max + base + u * kBlock + tid, base + u * kBlock + tid < total);
#pragma unroll
            for (int u = 0; u < 8; ++u) m = fmaxf(m, v[u]);
        }
        m = wave_max(m);
        if (lane == 0) l_max[wave] = m;
    }
    if (COUNT && tid < 64) {
        const int c = cb * 64 + tid;
        float gm = 0.0f, mu = 0.0f, sig = 0.0f;
        if (c < C) {
            fold_stats(ws, c, (double)N * (double)HW, gm, mu, sig);
            if (p == 0) { ws.gmax[c] = gm; ws.mean[c] = mu; ws.sigma[c] = sig; }
            if (EARLY) {
                const int guess = gm > ev.ratio * sig ? DAQ_CLASS_INVT : DAQ_CLASS_GAUSS;
                l_inv[tid] = inv_scale(clip_rule(guess, gm, s_state[c], ev.k, ev.A));
                if (p == 0) ws.pred[c] = (uint32_t)guess;
            }
        }
        // layer-wise clipping compares every element with the standard deviation of the whole tensor
        l_sigma[tid] = ws.scheme == DAQ_SCHEME_MCS ? ws.layer[2] : sig;
    }
    // forward pass (nothing is counted, the scale is given): the channel-major copy takes the same per-tensor scale
    if (!COUNT && EARLY && tid < 64) l_inv[tid] = inv_scale(sg);
    __syncthreads();
    if (!scale_ptr) sg = fmaxf(fmaxf(l_max[0], l_max[1]), fmaxf(l_max[2], l_max[3]));
    const float sg_raw = sg;
    if (!(sg >= kTinyScale)) sg = 0.0f;
    if (COUNT && blockIdx.x == 0) {
        // the clip state is overwritten by the packing pass: keep what this iteration started from
        for (int i = tid; i < C; i += kBlock) ws.s_prev[i] = s_state[i];
    }
    if (!scale_ptr && blockIdx.x == 0 && tid == 0) {
        *s_global = sg;
        ws.layer[0] = sg_raw;
    }
    // the NHWC buffer is a multiple of 256 bytes long: the bytes behind the last pixel hold no element and are zero
    if (WRITE_QG && blockIdx.x == 0 && tid < qg_tail) qg[(int64_t)M * c_pitch + tid] = 0;
    const float inv = inv_scale(sg);
    // sigma of the wave's 16 channels.  Lanes without a pixel and channels past C hold x = 0, and
    // 0 > sigma is false for every sigma >= 0, so the comparison needs no validity mask.
    // (both arrays are the same in every lane of the wave: moved to scalar registers, they cost no vector ones)
    auto uniform = [](float v) { return __uint_as_float((uint32_t)__builtin_amdgcn_readfirstlane((int)__float_as_uint(v))); };
    float sig[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) sig[i] = COUNT ? uniform(l_sigma[c0 - cb * 64 + i]) : 0.0f;

    float inv_c[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) inv_c[i] = EARLY ? uniform(l_inv[c0 - cb * 64 + i]) : 0.0f;

    uint32_t cnt[16];   // wave-uniform counters
#pragma unroll
    for (int i = 0; i < 16; ++i) cnt[i] = 0;
    for (int tile = t_first; tile < t_end; tile += t_step) {
        float nx[16];
        uint32_t n_nxt, px_nxt;
        bool v_nxt;
        fetch(tile + t_step, nx, n_nxt, px_nxt, v_nxt);
        uint32_t b[16], vb[16];
        const uint32_t idx0 = (n_cur * (uint32_t)C + (uint32_t)c0) * (uint32_t)HW + px_cur;   // the lane's 16 elements are one plane apart
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (COUNT) cnt[i] += (uint32_t)__popcll(__ballot(fabsf(x[i]) > sig[i]));
            const uint32_t idx = idx0 + (uint32_t)i * (uint32_t)HW;
            if (WRITE_QG) b[i] = quant_bits<STOCH>(x[i], inv, STOCH ? rng_u(seed, 1u, idx) : 0u);
            if (EARLY) vb[i] = quant_bits<STOCH>(x[i], inv_c[i], STOCH ? rng_u(seed, 0u, idx) : 0u);
        }
        if (EARLY) {
            // channel-major copy: the lane's pixel sits at the same offset of each of its 16 channel planes
            const uint32_t h = fdiv(px_cur, ev.div_w);
            int8_t* dst = ev.vq + (int64_t)c0 * ev.chan_pitch + (uint32_t)ev.lead +
                          (n_cur * (uint32_t)ev.img_rows + h) * (uint32_t)ev.row_pitch + (px_cur - h * (uint32_t)ev.W);
            if (ev.quad) {   // uniform
                // Four adjacent lanes hold four consecutive pixels of one row.  Their 4 x 16 codes are transposed inside
                // the quad - dwords between lanes, then bytes between dwords - so that lane r of the quad ends up with
                // the four pixels of channels 4r .. 4r+3 as one dword each: four stores per lane instead of sixteen.
                uint32_t wd[4];
#pragma unroll
                for (int k4 = 0; k4 < 4; ++k4) wd[k4] = pack4(vb[4 * k4], vb[4 * k4 + 1], vb[4 * k4 + 2], vb[4 * k4 + 3]);
                const bool o1 = lane & 1, o2 = lane & 2;
#pragma unroll
                for (int k4 = 0; k4 < 4; k4 += 2) {
                    const uint32_t got = quad_swap<true>(o1 ? wd[k4] : wd[k4 + 1]);
                    wd[k4] = o1 ? got : wd[k4];
                    wd[k4 + 1] = o1 ? wd[k4 + 1] : got;
                }
#pragma unroll
                for (int k4 = 0; k4 < 2; ++k4) {
                    const uint32_t got = quad_swap<false>(o2 ? wd[k4] : wd[k4 + 2]);
                    wd[k4] = o2 ? got : wd[k4];
                    wd[k4 + 2] = o2 ? wd[k4 + 2] : got;
                }
                // wd[q] = channels 4r .. 4r+3 of the quad's pixel q; now bytes: out[j] = pixels 0 .. 3 of channel 4r + j
                const uint32_t t0 = __builtin_amdgcn_perm(wd[1], wd[0], 0x05010400u), t1 = __builtin_amdgcn_perm(wd[1], wd[0], 0x07030602u);
                const uint32_t t2 = __builtin_amdgcn_perm(wd[3], wd[2], 0x05010400u), t3 = __builtin_amdgcn_perm(wd[3], wd[2], 0x07030602u);
                const uint32_t out[4] = {__builtin_amdgcn_perm(t2, t0, 0x05040100u), __builtin_amdgcn_perm(t2, t0, 0x07060302u),
                                         __builtin_amdgcn_perm(t3, t1, 0x05040100u), __builtin_amdgcn_perm(t3, t1, 0x07060302u)};
                const int r = lane & 3;
                int8_t* dq = dst - r + (int64_t)(4 * r) * ev.chan_pitch;   // first pixel of the quad, plane of channel c0 + 4r
                if (v_cur) {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (c0 + 4 * r + j < C) __builtin_memcpy(dq + (int64_t)j * ev.chan_pitch, &out[j], 4);   // byte aligned only
                }
            } else if (v_cur) {
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (c0 + i < C) dst[(int64_t)i * ev.chan_pitch] = (int8_t)vb[i];
            }
        }
        if (WRITE_QG && narrow) {
            const uint4 w = make_uint4(pack4(b[0], b[1], b[2], b[3]), pack4(b[4], b[5], b[6], b[7]),
                                       pack4(b[8], b[9], b[10], b[11]), pack4(b[12], b[13], b[14], b[15]));
            const uint32_t P = (uint32_t)(nsub * tile + sub) * kWave + lane;
            if (v_cur) *reinterpret_cast<uint4*>(qg + (int64_t)P * c_pitch + c0) = w;   // bytes of channels past C are codes of 0.0f: zeros
        } else if (WRITE_QG) {
            // A lane holds 16 channel bytes of ONE pixel, so a direct store would put 16 bytes into each of 64 different
            // lines.  The 64-pixel x 64-channel tile goes through LDS instead (80-byte pitch: conflict free both ways)
            // and leaves as whole 64-byte runs: four adjacent lanes write the 64 channel bytes of one pixel.
            const uint4 w = make_uint4(pack4(b[0], b[1], b[2], b[3]), pack4(b[4], b[5], b[6], b[7]),
                                       pack4(b[8], b[9], b[10], b[11]), pack4(b[12], b[13], b[14], b[15]));
            __syncthreads();   // the previous tile has been read out
            *reinterpret_cast<uint4*>(l_tile + lane * 80 + 16 * wave) = w;
            __syncthreads();
            const int opx = tid >> 2, och = 16 * (tid & 3);
            const uint32_t P = (uint32_t)tile * kWave + opx;   // pixels of a tile are consecutive in NHWC
            if (P < M && cb * 64 + och < c_pitch)
                *reinterpret_cast<uint4*>(qg + (int64_t)P * c_pitch + cb * 64 + och) =
                    *reinterpret_cast<const uint4*>(l_tile + opx * 80 + och);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = nx[i];
        n_cur = n_nxt; px_cur = px_nxt; v_cur = v_nxt;
    }
    if (COUNT) {
        uint32_t mine = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) mine = (lane == i) ? cnt[i] : mine;
        const bool mine_ok = lane < 16 && c0 + lane < C;
        if (narrow) {   // uniform: waves counted the same channels on different tiles
            uint32_t* l_c = reinterpret_cast<uint32_t*>(l_tile);
            if (lane < 16) l_c[16 * wave + lane] = mine;
            __syncthreads();
            if (sub == 0 && mine_ok) {
                uint32_t all = 0;
                for (int w = wave; w < 4; w += narrow) all += l_c[16 * w + lane];
                ws.part_cnt[(int64_t)(c0 + lane) * ws.cgroups + p] = all;
            }
        } else if (mine_ok) {
            ws.part_cnt[(int64_t)(c0 + lane) * ws.cgroups + p] = mine;
        }
        if (ws.scheme == DAQ_SCHEME_MCS) {   // uniform: one population; its count is the sum over all counting waves
            const uint32_t all = wave_sum_u32(mine_ok ? mine : 0u);
            if (lane == 0) ws.layer_cnt[blockIdx.x * (kBlock / kWave) + wave] = all;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Layer-wise Magnitude-aware Clipping (ablation study, the variant without vectorized quantization): the
// tensor is one population.  Two single-workgroup launches around the counting pass: before it, the statistics
// partials of all channels are folded into the tensor's mean and sigma (fixed summation order, so the result does
// not depend on the launch); after it, the counts of the counting waves into the tail mass, the class (Eq.
// "judge") and the clip value (Eq. "gaus" / Eq. "fats", with s_state[0] as the history).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_layer_stats(QuantWs ws, int C, double Mtot) {
    __shared__ double l_1[kBlock], l_2[kBlock];
    const int tid = threadIdx.x;
    double s1 = 0.0, s2 = 0.0;
    const int total = C * ws.slabs;
    for (int i = tid; i < total; i += kBlock) {
        s1 += ws.part_s1[i];
        s2 += ws.part_s2[i];
    }
    l_1[tid] = s1;
    l_2[tid] = s2;
    __syncthreads();
    for (int h = kBlock / 2; h > 0; h >>= 1) {
        if (tid < h) {
            l_1[tid] += l_1[tid + h];
            l_2[tid] += l_2[tid + h];
        }
        __syncthreads();
    }
    if (tid == 0) {
        const double mu = l_1[0] / Mtot;
        double var = l_2[0] / Mtot - mu * mu;
        if (var < 0.0) var = 0.0;
        ws.layer[1] = (float)mu;
        ws.layer[2] = (float)sqrt(var);
    }
}

__global__ __launch_bounds__(kBlock) void k_layer_decide(QuantWs ws, int waves, double Mtot, float k, float A, float lambda) {
    __shared__ uint32_t l_c[kBlock];
    const int tid = threadIdx.x;
    uint32_t cnt = 0;
    for (int base = 0; base < waves; base += 8 * kBlock) {   // eight loads in flight per thread
        uint32_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = base + u * kBlock + tid;
            v[u] = i < waves ? ws.layer_cnt[i] : 0u;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) cnt += v[u];
    }
    l_c[tid] = cnt;
    __syncthreads();
    for (int h = kBlock / 2; h > 0; h >>= 1) {
        if (tid < h) l_c[tid] += l_c[tid + h];
        __syncthreads();
    }
    if (tid == 0) {
        const double n = (double)l_c[0];
        const int klass = (n > (double)lambda * Mtot) ? DAQ_CLASS_GAUSS : DAQ_CLASS_INVT;
        ws.layer[3] = (float)(n / Mtot);
        ws.layer[4] = clip_rule(klass, ws.layer[0], ws.s_prev[0], k, A);
        ws.layer[5] = (float)klass;
    }
}

struct ClipArgs {
    float k, A, lambda;
    float* s_state;
    float* s_chan;
    uint8_t* cls;
    float* stats;
};

// ---------------------------------------------------------------------------------------------
// S5, channel-major copy: fp32 NCHW -> int8 CNHW (the dimension transformation G -> G', X -> X'),
// with S3 + S4 folded in for the per-channel copy of dY.
//
// Output driven: a workgroup produces 4096 consecutive bytes of one channel's plane, a thread four
// aligned dwords (256 dwords apart), including the zero bytes that serve as convolution padding, so
// every byte of the buffer is written exactly once, stores are 256-byte runs per wave and the loads
// of neighbouring lanes fall into the same cache lines.  All 16 loads of a thread are in flight
// before the scale is needed.
//
// CLIP: the scale is the channel's Magnitude-aware Clipping value.  Every workgroup of the channel
// sums the count partials of the counting pass, applies the discriminator (Eq. "judge") and the clip
// rule (Eq. "gaus" / Eq. "fats") to identical inputs in identical order, and the channel's first
// workgroup publishes s_chan, the class, the new state and the optional statistics.
// ---------------------------------------------------------------------------------------------
// S2 (sum of the count partials) + S3 discriminator + S4 clip rule for channel c, evaluated by a whole
// workgroup; every workgroup of the channel gets the same value, `publish` marks the one that writes it out.
__device__ __forceinline__ float clip_value(const QuantWs& ws, const ClipArgs& ca, int c, double Md, bool publish,
                                            uint32_t* l_cnt, int* klass_out = nullptr) {
    const int tid = threadIdx.x;
    if (ws.scheme == DAQ_SCHEME_MCS) {   // uniform: the layer's clip value, decided by k_layer_decide, for every channel
        const float s = ws.layer[4];
        if (klass_out) *klass_out = (int)ws.layer[5];
        if (publish && tid == 0) {
            ca.s_state[c] = s;
            ca.s_chan[c] = (s >= kTinyScale) ? s : 0.0f;
            ca.cls[c] = (uint8_t)ws.layer[5];
            if (ca.stats) {
                ca.stats[4 * c + 0] = ws.layer[0];
                ca.stats[4 * c + 1] = ws.layer[1];
                ca.stats[4 * c + 2] = ws.layer[2];
                ca.stats[4 * c + 3] = ws.layer[3];
            }
        }
        return s;
    }
    uint32_t cnt = 0;
    static_assert(kCountGrid <= 4 * kBlock, "a thread sums at most four count partials");
    {
        uint32_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = tid + u * kBlock;
            v[u] = __float_as_uint(ldf_or_zero(reinterpret_cast<const float*>(ws.part_cnt + (int64_t)c * ws.cgroups + i), i < ws.cgroups));
        }
        cnt = v[0] + v[1] + v[2] + v[3];
    }
    cnt = wave_sum_u32(cnt);
    if (tid % kWave == 0) l_cnt[tid / kWave] = cnt;
    __syncthreads();
    cnt = l_cnt[0] + l_cnt[1] + l_cnt[2] + l_cnt[3];
    const int klass = ((double)cnt > (double)ca.lambda * Md) ? DAQ_CLASS_GAUSS : DAQ_CLASS_INVT;
    if (klass_out) *klass_out = klass;   // every thread holds the same sum, hence the same class
    const float gm = ws.gmax[c];
    // ablation baselines: the tensor's |g|max for every channel (GQ) or the channel's own without clipping (GVQ);
    // class and statistics are reported as Algorithm 1 computes them
    const float s = ws.scheme == DAQ_SCHEME_GQ    ? ws.layer[0]
                    : ws.scheme == DAQ_SCHEME_GVQ ? gm
                                                  : clip_rule(klass, gm, ws.s_prev[c], ca.k, ca.A);
    if (publish && tid == 0) {
        ca.s_state[c] = s;
        ca.s_chan[c] = (s >= kTinyScale) ? s : 0.0f;
        ca.cls[c] = (uint8_t)klass;
        if (ca.stats) {
            ca.stats[4 * c + 0] = gm;
            ca.stats[4 * c + 1] = ws.mean[c];
            ca.stats[4 * c + 2] = ws.sigma[c];
            ca.stats[4 * c + 3] = (float)((double)cnt / Md);
        }
    }
    return s;
}

struct PackArgs {
    FastDiv div_slot, div_pitch;
    int per_chan;          // workgroups per (channel, phase) plane
    int lead_imgs;         // whole images that cover the leading zeros
    int per_channel_scale; // scale[c] instead of scale[0] (ignored with CLIP)
    uint32_t tensor;       // random stream id
    uint64_t seed;
};

template <typename T, bool STOCH, bool CLIP>
__global__ __launch_bounds__(kBlock) void k_pack_cnhw(const T* __restrict__ src, CnhwView L,
                                                      const float* __restrict__ scale, int8_t* __restrict__ dst,
                                                      PackArgs pa, QuantWs ws, ClipArgs ca) {
    __shared__ uint32_t l_cnt[kBlock / kWave];
    const int b = blockIdx.x;
    const int xcd = b % kXcd, q = b / kXcd;
    const int c = (q / pa.per_chan) * kXcd + xcd;  // channel c runs on XCD c % 8
    const int jb = q % pa.per_chan;                // block of 1024 dwords along the flattened axis
    const int phase = blockIdx.z;
    if (c >= L.C) return;
    const int tid = threadIdx.x;
    const int ph = phase / L.phases_w, pw = phase % L.phases_w;
    const int plane_dw = (int)(L.plane_pitch >> 2);
    const uint32_t slot = (uint32_t)(L.img_rows * L.row_pitch);
    const uint32_t HW = (uint32_t)(L.H * L.W);
    constexpr uint32_t EB = sizeof(T);   // bytes of a source element
    const __amdgpu_buffer_rsrc_t rs = f32_rsrc(src, (uint32_t)L.N * (uint32_t)L.C * HW * EB);

    // All index products below have factors under 2^24 and results under 2^31 (checked by the host), so the
    // full-rate 24-bit multiplier serves.  A destination row (n, r) reads source row h = r*phases_h + ph - org_h
    // of image n; stepping to the next destination row moves the source offset by one of two launch constants.
    const uint32_t W4 = (uint32_t)L.W * EB;
    const uint32_t step_row = (uint32_t)L.phases_h * W4;                                  // next row, same image
    const uint32_t step_img = (uint32_t)L.C * HW * EB - (uint32_t)(L.img_rows - 1) * step_row;  // row 0 of the next image
    const int h_first = ph - L.org_h, w_first = pw - L.org_w;

    float x[4][4];
    uint32_t eoff[4][4];   // byte offset of the element in the source (its index times the element size), or >= kOobOff
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int d = jb * 1024 + tid + 256 * u;   // dword inside the plane
        // first byte of the dword as (image, row, column); shifted by whole images so that the bytes in
        // front of the first image (the leading zeros) decompose to negative image numbers
        const uint32_t o = (uint32_t)(4 * d - (int)L.lead) + (uint32_t)pa.lead_imgs * slot;
        const uint32_t nq = fdiv(o, pa.div_slot);
        const uint32_t rem = o - __umul24(nq, slot);
        const uint32_t r = fdiv(rem, pa.div_pitch);
        const int col = (int)(rem - __umul24(r, (uint32_t)L.row_pitch));
        const int n = (int)nq - pa.lead_imgs;
        int h = (int)__umul24(r, (uint32_t)L.phases_h) + h_first;
        // n and h may be negative here (leading padding): signed multiplies keep the offset linear modulo 2^32,
        // so the row steps below land on the right value once the walk reaches a real row
        uint32_t raw = (uint32_t)(__mul24(__mul24(n, L.C) + c, (int)HW) + __mul24(h, L.W)) * EB;
        int w = (int)__umul24((uint32_t)col, (uint32_t)L.phases_w) + w_first;
        int nn = n, rr = (int)r, cc = col;
        const bool live = d < plane_dw;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bool ok = live & ((unsigned)nn < (unsigned)L.N) & ((unsigned)h < (unsigned)L.H) & ((unsigned)w < (unsigned)L.W);
            eoff[u][i] = ok ? raw + EB * (uint32_t)w : kOobOff;
            x[u][i] = buf_ld<T>(rs, eoff[u][i], 0u);
            // step to the next byte of the plane: next column, possibly next row, possibly next image
            const bool wrap = cc + 1 == L.row_pitch;
            const bool last = wrap & (rr + 1 == L.img_rows);
            cc = wrap ? 0 : cc + 1;
            w = wrap ? w_first : w + L.phases_w;
            raw += wrap ? (last ? step_img : step_row) : 0u;
            h = wrap ? (last ? h_first : h + L.phases_h) : h;
            rr = wrap ? (last ? 0 : rr + 1) : rr;
            nn += last ? 1 : 0;
        }
    }

    float s;
    if (CLIP) s = clip_value(ws, ca, c, (double)L.N * (double)L.H * (double)L.W, jb == 0 && phase == 0, l_cnt);
    else s = pa.per_channel_scale ? scale[c] : scale[0];
    const float inv = inv_scale(s);

    // Padding positions were read as 0.0f and quantize to code 0 in either rounding mode
    // (stochastic: floor(0) + (0 > u) = 0), so no select is needed here.
    int8_t* plane = dst + (int64_t)c * L.chan_pitch + (int64_t)phase * L.plane_pitch;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int d = jb * 1024 + tid + 256 * u;
        uint32_t bits[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            bits[i] = quant_bits<STOCH>(x[u][i], inv, STOCH ? rng_u(pa.seed, pa.tensor, eoff[u][i] / EB) : 0u);
        if (d < plane_dw) *reinterpret_cast<uint32_t*>(plane + 4 * (int64_t)d) = pack4(bits[0], bits[1], bits[2], bits[3]);
    }
}

// ---------------------------------------------------------------------------------------------
// S5, channel-major copy, fast path for unsplit layouts (one stride phase) whose row length is a
// multiple of V = 4 or 2.  Source driven: a thread loads V consecutive floats of one row with one
// aligned vector load (neighbouring lanes are contiguous: 1 KiB per wave instruction for V = 4),
// quantizes them and stores V consecutive bytes; no element needs a validity test and the index
// arithmetic is shared by V elements.  The zero bytes between the rows are written by the thread
// that owns the end of the row; the padding rows between images, the bytes in front of the first
// row and behind the last one by one extra workgroup per channel.  Every byte of the buffer is
// still written exactly once per call.
// ---------------------------------------------------------------------------------------------
struct RowsArgs {
    FastDiv div_hwv, div_wv, div_prb;
    int per_chan;          // blocks of 1024 element groups per channel
    int grid_per_chan;     // data workgroups per channel (one more zeroes the padding); fewer than per_chan: they loop
    int per_channel_scale;
    int early;             // the counting pass has written the real elements of channels whose class it guessed
    uint32_t tensor;
    uint64_t seed;
    // optional second copy of the same tensor in the same layout, quantized with its own per-tensor scale
    // (the globally quantized gradient of a depthwise layer): one read of the source serves both
    int8_t* dst2;
    const float* scale2;
    uint32_t tensor2;
};

template <int V>
__device__ __forceinline__ void store_codes(int8_t* p, uint32_t w) {
    // the destination has no alignment beyond one byte; the compiler picks the widest legal store
    if (V == 4) {
        __builtin_memcpy(p, &w, 4);
    } else {
        const uint16_t h = (uint16_t)w;
        __builtin_memcpy(p, &h, 2);
    }
}

template <typename T, bool STOCH, bool CLIP, int V>
__global__ __launch_bounds__(kBlock) void k_pack_rows(const T* __restrict__ src, CnhwView L,
                                                      const float* __restrict__ scale, int8_t* __restrict__ dst,
                                                      RowsArgs pa, QuantWs ws, ClipArgs ca) {
    __shared__ uint32_t l_cnt[kBlock / kWave];
    const int b = blockIdx.x;
    const int xcd = b % kXcd, q = b / kXcd;
    const int c = (q / (pa.grid_per_chan + 1)) * kXcd + xcd;  // channel c runs on XCD c % 8
    const int jb0 = q % (pa.grid_per_chan + 1);
    if (c >= L.C) return;
    const int tid = threadIdx.x;
    int8_t* plane = dst + (int64_t)c * L.chan_pitch;
    int8_t* plane2 = pa.dst2 ? pa.dst2 + (int64_t)c * L.chan_pitch : nullptr;   // uniform
    const uint32_t slot = (uint32_t)(L.img_rows * L.row_pitch);

    if (jb0 == pa.grid_per_chan) {
        // padding rows behind every image, then the bytes in front of the first row and behind the last image
        const uint32_t prb = (uint32_t)(L.img_rows - L.H) * (uint32_t)L.row_pitch;
        const uint32_t total = (uint32_t)L.N * prb;
        for (int copy = 0; copy < (plane2 ? 2 : 1); ++copy) {
            int8_t* pl = copy ? plane2 : plane;
            for (uint32_t t = tid; t < total; t += kBlock) {
                const uint32_t n = fdiv(t, pa.div_prb);
                pl[(uint32_t)L.lead + n * slot + (uint32_t)L.H * (uint32_t)L.row_pitch + (t - n * prb)] = 0;
            }
            for (uint32_t t = tid; t < (uint32_t)L.lead; t += kBlock) pl[t] = 0;
            for (uint32_t t = (uint32_t)L.lead + (uint32_t)L.N * slot + tid; t < (uint32_t)L.plane_pitch; t += kBlock) pl[t] = 0;
        }
        return;
    }

    // The counting pass guessed this channel's class: its bytes are in place if the guess was right (same clip rule
    // on the same inputs, hence the same scale and the same codes), and then nothing of dY is read here.
    float s = 0.0f;
    if (pa.early) {
        // the data workgroups of a correctly guessed channel return below: the zero bytes between the rows, which they
        // would have written along with the codes, are shared out among them first
        const uint32_t pw = (uint32_t)(L.row_pitch - L.W), rows = (uint32_t)L.N * (uint32_t)L.H;
        for (uint32_t t = (uint32_t)jb0 * kBlock + tid; t < rows * pw; t += (uint32_t)pa.grid_per_chan * kBlock) {
            const uint32_t r = t / pw, n = r / (uint32_t)L.H;
            const uint32_t at = (uint32_t)L.lead + (n * (uint32_t)L.img_rows + (r - n * (uint32_t)L.H)) * (uint32_t)L.row_pitch + (uint32_t)L.W + (t - r * pw);
            plane[at] = 0;
            if (plane2) plane2[at] = 0;
        }
        if constexpr (!CLIP) {
            return;   // a copy under a given scale (forward pass) is complete once its padding is written
        } else {
            int klass;
            s = clip_value(ws, ca, c, (double)L.N * (double)L.H * (double)L.W, jb0 == 0, l_cnt, &klass);
            if ((uint32_t)klass == ws.pred[c]) return;   // uniform
        }
    }
    if (CLIP && !pa.early) s = clip_value(ws, ca, c, (double)L.N * (double)L.H * (double)L.W, jb0 == 0, l_cnt);
    else if (!CLIP) s = pa.per_channel_scale ? scale[c] : scale[0];
    const float inv = inv_scale(s);

    const uint32_t HW = (uint32_t)(L.H * L.W), HWV = HW / V, WV = (uint32_t)L.W / V;
    const uint32_t groups = (uint32_t)L.N * HWV;
    const int padw = L.row_pitch - L.W;
    constexpr uint32_t EB = sizeof(T);   // bytes of a source element
    const __amdgpu_buffer_rsrc_t rs = f32_rsrc(src, (uint32_t)L.N * (uint32_t)L.C * HW * EB);

  // one pass unless the grid was cut down (early mode: the few channels left to do are walked by a few workgroups)
  for (int jb = jb0; jb < pa.per_chan; jb += pa.grid_per_chan) {
    float x[4][V];
    uint32_t eoff[4], doff[4];
    bool live[4], row_end[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const uint32_t gi = (uint32_t)jb * 1024u + tid + 256u * u;   // group of V elements inside the channel
        live[u] = gi < groups;
        const uint32_t gc = live[u] ? gi : 0u;
        const uint32_t n = fdiv(gc, pa.div_hwv);
        const uint32_t rem = gc - __umul24(n, HWV);
        const uint32_t h = fdiv(rem, pa.div_wv);
        const uint32_t wv = rem - __umul24(h, WV);
        row_end[u] = live[u] & (wv + 1 == WV);
        eoff[u] = live[u] ? __umul24(__umul24(n, (uint32_t)L.C) + (uint32_t)c, HW) * EB + rem * (EB * V) : kOobOff;
        doff[u] = (uint32_t)L.lead + __umul24(__umul24(n, (uint32_t)L.img_rows) + h, (uint32_t)L.row_pitch) + wv * V;
        if constexpr (EB == 4 && V == 4) {
            const v4u raw = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)eoff[u], 0, 0);
#pragma unroll
            for (int i = 0; i < V; ++i) x[u][i] = __uint_as_float(raw[i]);
        } else if constexpr (EB == 4) {
            const v2u raw = __builtin_amdgcn_raw_buffer_load_b64(rs, (int)eoff[u], 0, 0);
#pragma unroll
            for (int i = 0; i < V; ++i) x[u][i] = __uint_as_float(raw[i]);
        } else if constexpr (V == 4) {   // four bfloat16 in two dwords
            const v2u raw = __builtin_amdgcn_raw_buffer_load_b64(rs, (int)eoff[u], 0, 0);
            x[u][0] = __uint_as_float(raw[0] << 16);
            x[u][1] = __uint_as_float(raw[0] & 0xffff0000u);
            x[u][2] = __uint_as_float(raw[1] << 16);
            x[u][3] = __uint_as_float(raw[1] & 0xffff0000u);
        } else {                          // two bfloat16 in one dword
            const uint32_t raw = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rs, (int)eoff[u], 0, 0);
            x[u][0] = __uint_as_float(raw << 16);
            x[u][1] = __uint_as_float(raw & 0xffff0000u);
        }
    }

#pragma unroll
    for (int u = 0; u < 4; ++u) {
        uint32_t bits[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < V; ++i) bits[i] = quant_bits<STOCH>(x[u][i], inv, STOCH ? rng_u(pa.seed, pa.tensor, eoff[u] / EB + i) : 0u);
        if (live[u]) store_codes<V>(plane + doff[u], pack4(bits[0], bits[1], bits[2], bits[3]));
        if (row_end[u])
            for (int k = 0; k < padw; ++k) plane[doff[u] + V + k] = 0;
    }
    if (plane2) {
        const float inv2 = inv_scale(pa.scale2[0]);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            uint32_t bits[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int i = 0; i < V; ++i) bits[i] = quant_bits<STOCH>(x[u][i], inv2, STOCH ? rng_u(pa.seed, pa.tensor2, eoff[u] / EB + i) : 0u);
            if (live[u]) store_codes<V>(plane2 + doff[u], pack4(bits[0], bits[1], bits[2], bits[3]));
            if (row_end[u])
                for (int k = 0; k < padw; ++k) plane2[doff[u] + V + k] = 0;
        }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Channel-resident schedule: S1 - S5 for the per-channel copy with ONE read of dY.
//
// From the middle of a network on, a channel of the gradient is small (ResNet-50 at batch 64: 50176 elements at
// 28 x 28, 12544 at 14 x 14, 3136 at 7 x 7): the REGISTERS of one workgroup hold it.  One workgroup per channel
// loads its channel once and keeps it: statistics, tail mass, the discriminator's decision, the clip value and the
// per-channel quantization all run on registers.  The codes are assembled in an LDS image of the channel's plane
// (zero-filled first: the padding) and leave as whole 16-byte stores, so that every byte of the plane is written once.
// Only the globally quantized copy, whose scale is the maximum over ALL channels, needs a second launch (the counting
// kernel in its copy-only form), which finds a small tensor in the caches.
// ---------------------------------------------------------------------------------------------
constexpr int64_t kResidentMaxLds = 96 * 1024;   // bytes of a channel's int8 plane (the LDS image)

struct ResArgs {
    FastDiv div_hw, div_w;
    int N, C, HW;
    float k, A, lambda;
    uint64_t seed;         // the keys of stochastic rounding (round_keys)
};

// A load unit is four consecutive elements of one plane (VEC4: planes of a multiple of four elements in a 16-byte
// aligned fp32 tensor) or one element; a thread holds NU units, a workgroup has TH threads.
// FLAT (with VEC4): the plane has no padding between rows or images (1 x 1 layers), so element m of the channel sits at
// byte lead + m and a unit's four codes are one aligned dword of the plane: they go straight to memory, no LDS image.
template <typename T, bool STOCH, bool VEC4, int NU, int TH, bool FLAT = false>
__global__ __launch_bounds__(TH, NU <= 8 ? (VEC4 ? 6 : 8) : 4) void k_chan_resident(const T* __restrict__ g, CnhwView L, int8_t* __restrict__ vq,
                                                      ResArgs ra, QuantWs ws, ClipArgs ca) {
    extern __shared__ __align__(16) int8_t l_img[];   // the channel's plane as it will sit in memory
    __shared__ float l_mx[TH / kWave];
    __shared__ double l_s1[TH / kWave], l_s2[TH / kWave];
    __shared__ uint32_t l_cnt[TH / kWave];
    __shared__ float l_bc[4];   // |g|max, mean, sigma, clip value
    // workgroup b runs on XCD b % 8: an XCD takes a contiguous eighth of the channels, whose planes are neighbours in
    // every image and share cache lines where a plane is not a whole number of them
    const int per_xcd = (ra.C + kXcd - 1) / kXcd;
    const int c = ((int)blockIdx.x % kXcd) * per_xcd + (int)blockIdx.x / kXcd;
    if ((int)blockIdx.x / kXcd >= per_xcd || c >= ra.C) return;   // uniform: padding of the grid
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int HW = ra.HW, M = ra.N * HW;
    constexpr uint32_t EB = sizeof(T);
    constexpr int PER = VEC4 ? 4 : 1;
    const __amdgpu_buffer_rsrc_t rs = f32_rsrc(g, (uint32_t)M * (uint32_t)ra.C * EB);
    const int units = (M + PER - 1) / PER;
    const uint32_t skip = (uint32_t)(ra.C - 1) * (uint32_t)HW, first = (uint32_t)c * (uint32_t)HW;   // the other channels' planes of an image

    // ---- S1: the channel comes in, all loads of the thread in flight at once ----
    float x[NU][PER];
#pragma unroll
    for (int u = 0; u < NU; ++u) {
        const int q = u * TH + tid;
        const bool ok = q < units;
        const uint32_t m = ok ? (uint32_t)q * PER : 0u;
        const uint32_t n = fdiv(m, ra.div_hw);
        const uint32_t off = ok ? (m + n * skip + first) * EB : kOobOff;   // NCHW index (n*C + c)*HW + (m - n*HW)
        if constexpr (VEC4) {
            const v4u raw = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)off, 0, 0);
#pragma unroll
            for (int e = 0; e < 4; ++e) x[u][e] = __uint_as_float(raw[e]);
        } else {
            x[u][0] = buf_ld<T>(rs, off, 0u);
        }
    }
    if constexpr (STOCH) __builtin_amdgcn_sched_barrier(0);   // every load of the channel is requested before the hashes below start
    // Stochastic rounding: an element's draw depends on its index alone, so the hashes are computed here, while the
    // loads are on their way and the vector ALU has nothing else to do, and kept as 16-bit halves (element k of the
    // thread in half k % 2 of word k / 2).
    uint32_t draw[STOCH ? (NU * PER + 1) / 2 : 1];
    if constexpr (STOCH) {
#pragma unroll
        for (int k = 0; k < NU * PER; k += 2) {
            uint32_t h[2] = {0u, 0u};
#pragma unroll
            for (int t = 0; t < 2 && k + t < NU * PER; ++t) {
                const int u = (k + t) / PER, e = (k + t) % PER;
                const uint32_t m = (uint32_t)(u * TH + tid) * PER;   // (units past the channel hash a number nobody uses)
                const uint32_t n = fdiv(m, ra.div_hw);
                h[t] = fmix32((m + n * skip + first + (uint32_t)e) ^ (uint32_t)ra.seed);
            }
            draw[k / 2] = (h[0] >> 16) | (h[1] & 0xffff0000u);   // the per-channel copy draws from the upper half of the hash
        }
        // (without this the compiler moves the hashes down to where they are used, behind the barriers; as many of
        // them as the registers of the form allow)
        constexpr int W = (NU * PER + 1) / 2;
        constexpr int PIN = NU <= 8 ? (FLAT || !VEC4 ? W : W / 2) : FLAT ? 3 * W / 4 : W / 2;
#pragma unroll
        for (int k = 0; k < PIN; ++k) asm volatile("" : "+v"(draw[k]));
        __builtin_amdgcn_sched_barrier(0);
    }
    auto draw_of = [&](int u, int e) -> uint32_t {
        if constexpr (!STOCH) return 0u;
        const int k = u * PER + e;
        return (k & 1) ? draw[k / 2] >> 16 : draw[k / 2] & 0xffffu;
    };
    float mx = 0.0f;
    double s1 = 0.0, s2 = 0.0;
#pragma unroll
    for (int u = 0; u < NU; ++u)
#pragma unroll
        for (int e = 0; e < PER; ++e) {   // units past the channel were read as zeros and change nothing
            mx = fmaxf(mx, fabsf(x[u][e]));
            const double a = x[u][e];
            s1 += a;
            s2 = __builtin_fma(a, a, s2);   // the square of a widened fp32 is exact in fp64: the same sum as s2 + a * a, one instruction
        }
    mx = wave_max(mx);
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    if (lane == 0) { l_mx[wave] = mx; l_s1[wave] = s1; l_s2[wave] = s2; }
    // the padding of the plane image, while the partials settle
    if constexpr (!FLAT)
        for (int i = tid; i < (int)(L.plane_pitch >> 4); i += TH) reinterpret_cast<uint4*>(l_img)[i] = make_uint4(0u, 0u, 0u, 0u);
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < TH / kWave; ++w) { mx = fmaxf(mx, l_mx[w]); s1 += l_s1[w]; s2 += l_s2[w]; }
        const double Md = (double)ra.N * (double)HW;
        const double mu = s1 / Md;
        double var = s2 / Md - mu * mu;
        if (var < 0.0) var = 0.0;
        l_bc[0] = mx;
        l_bc[1] = (float)mu;
        l_bc[2] = (float)sqrt(var);
    }
    __syncthreads();
    const float gm = l_bc[0], sigma = l_bc[2];

    // ---- S2: tail mass (a zero never exceeds sigma, so the units past the channel need no mask) ----
    uint32_t cnt = 0;   // of the whole wave: a scalar counter
#pragma unroll
    for (int u = 0; u < NU; ++u)
#pragma unroll
        for (int e = 0; e < PER; ++e) cnt += (uint32_t)__popcll(__ballot(fabsf(x[u][e]) > sigma));
    if (lane == 0) l_cnt[wave] = cnt;
    __syncthreads();
    if (tid == 0) {
        // S3 + S4: discriminator (Eq. "judge") and clip value (Eq. "gaus" / Eq. "fats"), then what the channel publishes
        for (int w = 1; w < TH / kWave; ++w) cnt += l_cnt[w];
        const double Md = (double)ra.N * (double)HW;
        const int klass = ((double)cnt > (double)ra.lambda * Md) ? DAQ_CLASS_GAUSS : DAQ_CLASS_INVT;
        const float sc = clip_rule(klass, gm, ca.s_state[c], ra.k, ra.A);
        l_bc[3] = sc;
        ca.s_state[c] = sc;
        ca.s_chan[c] = (sc >= kTinyScale) ? sc : 0.0f;
        ca.cls[c] = (uint8_t)klass;
        if (ca.stats) {
            ca.stats[4 * c + 0] = gm;
            ca.stats[4 * c + 1] = l_bc[1];
            ca.stats[4 * c + 2] = sigma;
            ca.stats[4 * c + 3] = (float)((double)cnt / Md);
        }
        ws.part_max[c] = gm;   // one partial per channel: the copy-only launch folds them into the global scale
    }
    __syncthreads();
    const float inv = inv_scale(l_bc[3]);

    if constexpr (FLAT) {
        // ---- S5, plane without padding: a unit's four codes are dword q of the plane's payload ----
        uint32_t* plane32 = reinterpret_cast<uint32_t*>(vq + (int64_t)c * L.chan_pitch);   // chan_pitch is a multiple of 256
        uint32_t* pay = plane32 + (L.lead >> 2);
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int q = u * TH + tid;
            if (q < units) {
                uint32_t b[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) b[e] = quant_bits<STOCH>(x[u][e], inv, draw_of(u, e));
                pay[q] = pack4(b[0], b[1], b[2], b[3]);
            }
        }
        // the zeros in front of and behind the payload
        const int head = (int)(L.lead >> 2), tail = head + units, total = (int)(L.plane_pitch >> 2);
        for (int i = tid; i < head; i += TH) plane32[i] = 0u;
        for (int i = tail + tid; i < total; i += TH) plane32[i] = 0u;
        return;
    }
    // ---- S5: the per-channel codes go to their places in the plane image ----
    const uint32_t slot = (uint32_t)(L.img_rows * L.row_pitch);
#pragma unroll
    for (int u = 0; u < NU; ++u) {
        const int q = u * TH + tid;
        if (q < units) {
            const uint32_t m = (uint32_t)q * PER;
            const uint32_t n = fdiv(m, ra.div_hw);
            const uint32_t px = m - n * (uint32_t)HW;
            uint32_t r = fdiv(px, ra.div_w);
            uint32_t col = px - r * (uint32_t)L.W;
            uint32_t pos = (uint32_t)L.lead + n * slot + r * (uint32_t)L.row_pitch + col;
#pragma unroll
            for (int e = 0; e < PER; ++e) {
                l_img[pos] = (int8_t)quant_bits<STOCH>(x[u][e], inv, draw_of(u, e));
                const bool wrap = ++col == (uint32_t)L.W;   // a unit stays inside its image, but may run on into the next row
                col = wrap ? 0u : col;
                pos += wrap ? (uint32_t)(L.row_pitch - L.W) + 1u : 1u;
            }
        }
    }
    __syncthreads();
    uint4* plane = reinterpret_cast<uint4*>(vq + (int64_t)c * L.chan_pitch);   // chan_pitch is a multiple of 256
    for (int i = tid; i < (int)(L.plane_pitch >> 4); i += TH) plane[i] = reinterpret_cast<const uint4*>(l_img)[i];
}

// ---------------------------------------------------------------------------------------------
// per-tensor helpers for the forward pass
// ---------------------------------------------------------------------------------------------
// max |x| of a tensor into *bits (the bit pattern of a non-negative float orders like the float).  One atomic per
// workgroup: atomics on one address are served one after the other (about 10 ns each), so a kernel that ends every
// wave with one spends longer on them than on the tensor.  16-byte loads, four in flight per thread.
__global__ __launch_bounds__(kBlock) void k_absmax(const float* __restrict__ x, int64_t n, uint32_t* bits) {
    __shared__ float l_m[kBlock / kWave];
    float m = 0.0f;
    const int64_t n4 = ((uintptr_t)x & 15u) ? 0 : n / 4;   // whole aligned quads; the rest goes element by element
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    const float4* x4 = reinterpret_cast<const float4*>(x);
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    for (; i + 3 * stride < n4; i += 4 * stride) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = x4[i + u * stride];
#pragma unroll
        for (int u = 0; u < 4; ++u) m = fmaxf(m, fmaxf(fmaxf(fabsf(v[u].x), fabsf(v[u].y)), fmaxf(fabsf(v[u].z), fabsf(v[u].w))));
    }
    for (; i < n4; i += stride) {
        const float4 v = x4[i];
        m = fmaxf(m, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
    }
    for (int64_t j = 4 * n4 + (int64_t)blockIdx.x * kBlock + threadIdx.x; j < n; j += stride) m = fmaxf(m, fabsf(x[j]));
    m = wave_max(m);
    if (threadIdx.x % kWave == 0) l_m[threadIdx.x / kWave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kBlock / kWave; ++w) m = fmaxf(m, l_m[w]);
        atomicMax(bits, __float_as_uint(m));
    }
}

// Scale of the per-tensor copy from the per-channel maxima of the channel-resident pass (one workgroup).
__global__ __launch_bounds__(kBlock) void k_fold_max(QuantWs ws, int C, float* __restrict__ s_global) {
    __shared__ float l_m[kBlock / kWave];
    float m = 0.0f;
    for (int i = threadIdx.x; i < C; i += kBlock) m = fmaxf(m, ws.part_max[i]);
    m = wave_max(m);
    if (threadIdx.x % kWave == 0) l_m[threadIdx.x / kWave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        m = fmaxf(fmaxf(l_m[0], l_m[1]), fmaxf(l_m[2], l_m[3]));
        ws.layer[0] = m;
        *s_global = (m >= kTinyScale) ? m : 0.0f;
    }
}

__global__ void k_scale_from_bits(const uint32_t* bits, float* s) {
    const float v = __uint_as_float(*bits);
    *s = (v >= kTinyScale) ? v : 0.0f;
}

// q(W) in its three arrangements (see daq_wpack_layout); the buffer is zero-filled beforehand.
__global__ __launch_bounds__(kBlock) void k_pack_w(const float* __restrict__ W, const float* __restrict__ s_w,
                                                   int Cout, int Cin, int groups, int kH, int kW,
                                                   daq_wpack_layout L, int8_t* __restrict__ out) {
    const int cig = Cin / groups, cog = Cout / groups, taps = kH * kW;
    const int64_t total = (int64_t)Cout * cig * taps;
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    const int tap = (int)(i % taps);
    const int cl = (int)((i / taps) % cig);
    const int co = (int)(i / ((int64_t)taps * cig));
    const int g = co / cog, col = co % cog;
    const int ci = g * cig + cl;
    const float inv = inv_scale(*s_w);
    const int8_t code = (int8_t)quant_code<false>(W[i], inv, 0u);
    out[L.off_plain + i] = code;
    out[L.off_fwd + ((int64_t)tap * Cout + co) * L.cig_pitch + cl] = code;
    out[L.off_bwd + ((int64_t)tap * Cin + ci) * L.cog_pitch + col] = code;
    if (groups == 1) {
        // fragment order: element (tap, row, k) of a copy with RB row blocks
        auto frag = [&](int row, int k, int RB) -> int64_t {
            return ((((int64_t)(k >> 6) * taps + tap) * RB + (row >> 5)) * 2 + ((k & 63) >> 5)) * 1024 +
                   ((((k & 31) >> 4) * 32 + (row & 31)) * 16) + (k & 15);
        };
        out[L.off_fwd_frag + frag(co, ci, (Cout + 31) / 32)] = code;
        out[L.off_bwd_frag + frag(ci, co, (Cin + 31) / 32)] = code;
    }
}

// grid of k_pack_cnhw: x enumerates (channel, block of 1024 dwords) with the channel's XCD in the low bits,
// z the stride phase
int pack_per_chan(const daq_layout& L) { return (int)ceil_div(L.plane_pitch / 4, 4 * kBlock); }
dim3 pack_grid(const daq_layout& L) {
    return dim3((unsigned)(round_up(L.C, kXcd) * pack_per_chan(L)), 1u, (unsigned)(L.phases_h * L.phases_w));
}
PackArgs pack_args(const daq_layout& L, int per_channel_scale, uint32_t tensor, uint64_t seed) {
    PackArgs pa{};
    pa.div_slot = make_fastdiv((uint32_t)(L.img_rows * L.row_pitch));
    pa.div_pitch = make_fastdiv((uint32_t)L.row_pitch);
    pa.per_chan = pack_per_chan(L);
    pa.lead_imgs = (int)ceil_div(L.lead, (int64_t)L.img_rows * L.row_pitch);
    pa.per_channel_scale = per_channel_scale;
    pa.tensor = tensor;
    pa.seed = seed;
    return pa;
}
// The packing kernel indexes a plane with 32-bit integers.
bool pack_supported(const daq_layout& L) {
    const int64_t lim24 = (int64_t)1 << 24;
    return L.plane_pitch + L.lead + (int64_t)L.img_rows * L.row_pitch < ((int64_t)1 << 31) && (L.plane_pitch & 3) == 0 &&
           (int64_t)L.img_rows * L.row_pitch < lim24 &&
           (int64_t)(L.N + 1 + ceil_div(L.lead, (int64_t)L.img_rows * L.row_pitch)) * L.C < lim24 / 2 && (int64_t)L.H * L.W < lim24 / 2 &&
           (int64_t)L.img_rows * L.phases_h < lim24 && (int64_t)L.row_pitch * L.phases_w < lim24;
}
// The quantization kernels read an fp32 tensor through a buffer descriptor with 32-bit offsets.
bool f32_tensor_supported(int64_t elems) { return elems * 4 < ((int64_t)1 << 31); }


// Bytes of an NHWC buffer behind its last pixel (the buffer is rounded up to 256 bytes).
int nhwc_tail(const daq_layout& L) { return (int)(L.bytes - (int64_t)L.N * L.H * L.W * L.c_pitch); }

// Elements per thread of the source-driven row kernel (4 or 2), or 0 when the layout needs the output-driven one.
int rows_vector(const daq_layout& Ld, const void* src, int elem_bytes = 4) {
    const int64_t lim24 = (int64_t)1 << 24;
    const bool unsplit = Ld.phases_h == 1 && Ld.phases_w == 1 && Ld.org_h == 0 && Ld.org_w == 0 &&
                         (int64_t)Ld.N * Ld.img_rows < lim24 && (int64_t)Ld.H * Ld.W < lim24 &&
                         (int64_t)(Ld.N + 1) * Ld.C < lim24 && Ld.plane_pitch < ((int64_t)1 << 31);
    // the vector of 4 or 2 source elements a thread loads must be aligned as a whole
    if (unsplit && Ld.W % 4 == 0 && ((uintptr_t)src & (uintptr_t)(4 * elem_bytes - 1)) == 0) return 4;
    if (unsplit && Ld.W % 2 == 0 && ((uintptr_t)src & (uintptr_t)(2 * elem_bytes - 1)) == 0) return 2;
    return 0;
}

// Launches the channel-major packing of one fp32 NCHW tensor: the source-driven row kernel when the
// layout allows it, the output-driven kernel otherwise.
// With dst2 the same pass also writes a second copy quantized with the per-tensor scale scale2 (random stream
// tensor2); *fused tells whether that happened - the output-driven kernel writes one copy per launch.
template <typename T>
daq_status launch_pack(const char* name, bool stoch, bool clip, const T* src, const daq_layout& Ld,
                       const float* scale, int per_channel_scale, int8_t* dst, uint32_t tensor, uint64_t seed,
                       const QuantWs& ws, const ClipArgs& ca, hipStream_t st, int8_t* dst2 = nullptr,
                       const float* scale2 = nullptr, uint32_t tensor2 = 0, bool* fused = nullptr, bool early = false) {
    if (fused) *fused = false;
    const CnhwView V = cnhw_view(Ld);
    const int v = rows_vector(Ld, src, (int)sizeof(T));
    if (early && !v) return DAQ_ERR_INVALID_ARG;   // the caller checks rows_vector before it asks for the early copy
    if (v) {
        RowsArgs ra{};
        const uint32_t hwv = (uint32_t)(Ld.H * Ld.W / v);
        ra.div_hwv = make_fastdiv(hwv);
        ra.div_wv = make_fastdiv((uint32_t)(Ld.W / v));
        ra.div_prb = make_fastdiv((uint32_t)std::max(1, (Ld.img_rows - Ld.H) * Ld.row_pitch));
        ra.per_chan = (int)ceil_div((int64_t)Ld.N * hwv, 4 * kBlock);
        ra.grid_per_chan = early ? std::min(ra.per_chan, 16) : ra.per_chan;
        ra.per_channel_scale = per_channel_scale;
        ra.early = early ? 1 : 0;
        ra.tensor = tensor;
        ra.seed = seed;
        ra.dst2 = dst2;
        ra.scale2 = scale2;
        ra.tensor2 = tensor2;
        if (fused) *fused = dst2 != nullptr;
        const dim3 grid((unsigned)(round_up(Ld.C, kXcd) * (ra.grid_per_chan + 1)));
#define DAQ_ROWS(S, CL, VV) \
    DAQ_LAUNCH(name, st, hipLaunchKernelGGL((k_pack_rows<T, S, CL, VV>), grid, dim3(kBlock), 0, st, src, V, scale, dst, ra, ws, ca))
        if (v == 4) {
            if (stoch) { if (clip) DAQ_ROWS(true, true, 4); else DAQ_ROWS(true, false, 4); }
            else { if (clip) DAQ_ROWS(false, true, 4); else DAQ_ROWS(false, false, 4); }
        } else {
            if (stoch) { if (clip) DAQ_ROWS(true, true, 2); else DAQ_ROWS(true, false, 2); }
            else { if (clip) DAQ_ROWS(false, true, 2); else DAQ_ROWS(false, false, 2); }
        }
#undef DAQ_ROWS
        return DAQ_OK;
    }
    if (!pack_supported(Ld)) return DAQ_ERR_UNSUPPORTED;
    const PackArgs pa = pack_args(Ld, per_channel_scale, tensor, seed);
    const dim3 grid = pack_grid(Ld);
#define DAQ_PACK(S, CL) \
    DAQ_LAUNCH(name, st, hipLaunchKernelGGL((k_pack_cnhw<T, S, CL>), grid, dim3(kBlock), 0, st, src, V, scale, dst, pa, ws, ca))
    if (stoch) { if (clip) DAQ_PACK(true, true); else DAQ_PACK(true, false); }
    else { if (clip) DAQ_PACK(false, true); else DAQ_PACK(false, false); }
#undef DAQ_PACK
    return DAQ_OK;
}

}  // namespace

size_t quantize_grad_ws_bytes(const daq_conv_desc& d) {
    return (size_t)carve_quant_ws(nullptr, d.Cout, d.N, daq_out_h(&d) * daq_out_w(&d)).total_bytes;
}

size_t fwd_quant_ws_bytes(const daq_conv_desc&) { return 256; }

// ---------------------------------------------------------------------------------------------
// forward-side quantization of X (two layouts) and W (packed)
// ---------------------------------------------------------------------------------------------
// Whether the forward pass can quantize this activation: everything that could fail is decided here, before the
// first launch, so that an unsupported problem leaves every output untouched.
daq_status quantize_activation_check(const daq_conv_desc& d, const float* X) {
    daq_layout Ln, Lc;
    if (daq_layout_qx_nhwc(&d, &Ln) != DAQ_OK || daq_layout_qx_cnhw(&d, &Lc) != DAQ_OK) return DAQ_ERR_INVALID_ARG;
    if (!f32_tensor_supported((int64_t)d.N * d.Cin * d.Hin * d.Win)) return DAQ_ERR_UNSUPPORTED;
    if (rows_vector(Lc, X) == 0 && !pack_supported(Lc)) return DAQ_ERR_UNSUPPORTED;
    return DAQ_OK;
}

daq_status quantize_activation(const daq_conv_desc& d, const float* X, int8_t* qx_nhwc, int8_t* qx_cnhw, float* s_x,
                               void* wsp, hipStream_t st, daq_schedule schedule) {
    const daq_status ok = quantize_activation_check(d, X);
    if (ok != DAQ_OK) return ok;
    uint32_t* bits = (uint32_t*)wsp;
    const int64_t n = (int64_t)d.N * d.Cin * d.Hin * d.Win;
    DAQ_LAUNCH("fill", st, hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, st, bits, (int64_t)1, 0u));
    const int blocks = (int)std::min<int64_t>(ceil_div(n, kBlock * 16), 1024);
    DAQ_LAUNCH("absmax", st, hipLaunchKernelGGL(k_absmax, dim3(blocks), dim3(kBlock), 0, st, X, n, bits));
    DAQ_LAUNCH("scale", st, hipLaunchKernelGGL(k_scale_from_bits, dim3(1), dim3(1), 0, st, bits, s_x));

    daq_layout Ln, Lc;
    if (daq_layout_qx_nhwc(&d, &Ln) != DAQ_OK || daq_layout_qx_cnhw(&d, &Lc) != DAQ_OK) return DAQ_ERR_INVALID_ARG;
    const int HW = d.Hin * d.Win;
    const int CB = (int)ceil_div(d.Cin, 64);
    QuantWs geo = carve_quant_ws(nullptr, d.Cin, d.N, HW);  // only the tile geometry is used: nothing is counted here
    // Unit-stride layers whose channel-major layout the row kernel serves: one sweep over X writes both copies (the
    // mechanism of the early per-channel copy of dY, with the per-tensor scale), then the padding bytes are filled in.
    // (by default from 8 Mi elements on: below that the two lean passes are faster, as for dY)
    const bool want_early = schedule == DAQ_SCHEDULE_EARLY_COPY || (schedule == DAQ_SCHEDULE_AUTO && n >= ((int64_t)8 << 20));
    if (want_early && rows_vector(Lc, X) != 0 && Lc.lead + (int64_t)d.N * Lc.img_rows * Lc.row_pitch < ((int64_t)1 << 32)) {
        const EarlyVq ev{qx_cnhw, Lc.chan_pitch, (int32_t)Lc.lead, Lc.img_rows, Lc.row_pitch, Lc.W, make_fastdiv((uint32_t)Lc.W),
                         0.0f, 0.0f, 0.0f, Lc.W % 4 == 0 ? 1 : 0};
        DAQ_LAUNCH("quant_both", st,
                   hipLaunchKernelGGL((k_count_qg<float, false, true, false, true>), dim3(CB * geo.cgroups), dim3(kBlock), 0, st, X,
                                      d.N, d.Cin, HW, Ln.c_pitch, make_fastdiv((uint32_t)HW), geo, (const float*)s_x, qx_nhwc,
                                      (uint64_t)0, (const float*)nullptr, (float*)nullptr, ev, nhwc_tail(Ln)));
        return launch_pack("pad_cnhw", false, false, X, Lc, (const float*)s_x, 0, qx_cnhw, 0u, 0, geo, ClipArgs{}, st, nullptr, nullptr,
                           0, nullptr, true);
    }
    DAQ_LAUNCH("quant_nhwc", st,
               hipLaunchKernelGGL((k_count_qg<float, false, true, false>), dim3(CB * geo.cgroups), dim3(kBlock), 0, st, X, d.N,
                                  d.Cin, HW, Ln.c_pitch, make_fastdiv((uint32_t)HW), geo, (const float*)s_x, qx_nhwc,
                                  (uint64_t)0, (const float*)nullptr, (float*)nullptr, EarlyVq{}, nhwc_tail(Ln)));
    const daq_status prc = launch_pack("pack_cnhw", false, false, X, Lc, (const float*)s_x, 0, qx_cnhw, 0u, 0, geo, ClipArgs{}, st);
    if (prc != DAQ_OK) return prc;
    return DAQ_OK;
}

daq_status quantize_filter(const daq_conv_desc& d, const float* W, int8_t* qw, float* s_w, void* wsp,
                           hipStream_t st) {
    uint32_t* bits = (uint32_t*)wsp + 16;
    daq_wpack_layout L;
    if (daq_layout_qw(&d, &L) != DAQ_OK) return DAQ_ERR_INVALID_ARG;
    const int64_t n = (int64_t)d.Cout * (d.Cin / d.groups) * d.kH * d.kW;
    DAQ_LAUNCH("fill", st, hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, st, bits, (int64_t)1, 0u));
    DAQ_LAUNCH("fill", st,
               hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)ceil_div(L.bytes / 4, kBlock)), dim3(kBlock), 0, st,
                                  (uint32_t*)qw, L.bytes / 4, 0u));
    const int blocks = (int)std::min<int64_t>(ceil_div(n, kBlock * 16), 1024);
    DAQ_LAUNCH("absmax", st, hipLaunchKernelGGL(k_absmax, dim3(blocks), dim3(kBlock), 0, st, W, n, bits));
    DAQ_LAUNCH("scale", st, hipLaunchKernelGGL(k_scale_from_bits, dim3(1), dim3(1), 0, st, bits, s_w));
    DAQ_LAUNCH("pack_w", st,
               hipLaunchKernelGGL(k_pack_w, dim3((unsigned)ceil_div(n, kBlock)), dim3(kBlock), 0, st, W,
                                  (const float*)s_w, d.Cout, d.Cin, d.groups, d.kH, d.kW, L, qw));
    return DAQ_OK;
}

}  // namespace daq

using namespace daq;

// ---------------------------------------------------------------------------------------------
// Algorithm 1, per-channel loop + vectorized and global quantization
// ---------------------------------------------------------------------------------------------
namespace {

// Orders everything launched on `later` from now on behind everything launched on `first` so far.  One event per
// device, created on first use and kept: a wait refers to the state of the event at the time of the call, so the
// next record does not disturb it.
daq_status stream_follows(hipStream_t later, hipStream_t first) {
    static std::mutex mu;
    static hipEvent_t ev[64] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return DAQ_ERR_HIP;
    std::lock_guard<std::mutex> lock(mu);
    if (!ev[dev] && hipEventCreateWithFlags(&ev[dev], hipEventDisableTiming) != hipSuccess) return DAQ_ERR_HIP;
    if (hipEventRecord(ev[dev], first) != hipSuccess || hipStreamWaitEvent(later, ev[dev], 0) != hipSuccess) return DAQ_ERR_HIP;
    return DAQ_OK;
}

// Per-channel statistics that the producer of dY already has (S1 of Algorithm 1): |g|max, sum and sum of squares.
struct ProducerStats {
    const float* absmax;
    const double* sum;
    const double* sumsq;
};

// T = float or uint16_t (bfloat16): the element type of dY
template <typename T>
daq_status quantize_grad_impl(const daq_conv_desc* desc, const T* dY, float* s_state, float k, float A, float lambda,
                              daq_round mode, uint64_t seed, daq_scheme scheme, daq_schedule schedule, int8_t* vq,
                              int8_t* qg, float* s_chan, float* s_global, uint8_t* cls, float* stats, void* workspace,
                              size_t workspace_bytes, void* stream, void* side_stream = nullptr,
                              const ProducerStats* given = nullptr) {
    if (!desc_valid(desc) || !dY || !s_state || !vq || !qg || !s_chan || !s_global || !cls)
        return DAQ_ERR_INVALID_ARG;
    if (given && (!given->absmax || !given->sum || !given->sumsq || ((uintptr_t)given->absmax & 3u) ||
                  ((uintptr_t)given->sum & 7u) || ((uintptr_t)given->sumsq & 7u)))
        return DAQ_ERR_INVALID_ARG;
    if (mode != DAQ_ROUND_NEAREST && mode != DAQ_ROUND_STOCHASTIC) return DAQ_ERR_INVALID_ARG;
    if (scheme != DAQ_SCHEME_DAQ && scheme != DAQ_SCHEME_GQ && scheme != DAQ_SCHEME_GVQ && scheme != DAQ_SCHEME_MCS)
        return DAQ_ERR_INVALID_ARG;
    if (schedule != DAQ_SCHEDULE_AUTO && schedule != DAQ_SCHEDULE_THREE_SWEEPS && schedule != DAQ_SCHEDULE_EARLY_COPY &&
        schedule != DAQ_SCHEDULE_CHANNEL_RESIDENT)
        return DAQ_ERR_INVALID_ARG;
    if (((uintptr_t)dY & (sizeof(T) - 1)) || ((uintptr_t)vq & 15u) || ((uintptr_t)qg & 15u)) return DAQ_ERR_INVALID_ARG;
    daq_layout Lv, Lg;
    daq_status rc = daq_layout_vq(desc, &Lv);
    if (rc != DAQ_OK) return rc;
    rc = daq_layout_qg(desc, &Lg);
    if (rc != DAQ_OK) return rc;
    const size_t need = daq_workspace_bytes(DAQ_OP_QUANTIZE_GRAD, desc);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u)) return DAQ_ERR_WORKSPACE;

    // the kernels address dY with 32-bit byte offsets
    if (!((int64_t)desc->N * desc->Cout * daq_out_h(desc) * daq_out_w(desc) * (int64_t)sizeof(T) < ((int64_t)1 << 31)))
        return DAQ_ERR_UNSUPPORTED;
    // the packing pass is the last launch: what it cannot serve is refused here, before the first one
    if (rows_vector(Lv, dY, (int)sizeof(T)) == 0 && !pack_supported(Lv)) return DAQ_ERR_UNSUPPORTED;

    hipStream_t st = (hipStream_t)stream;
    // With a side stream, what only the filter gradient consumes leaves the stream of the data gradient: from the
    // point where qg and s_global need nothing more, the side stream waits for `st` and takes the remaining launches.
    hipStream_t side = (side_stream && side_stream != stream) ? (hipStream_t)side_stream : nullptr;
    const int N = desc->N, C = desc->Cout, Ho = daq_out_h(desc), Wo = daq_out_w(desc);
    const int HW = Ho * Wo;
    const bool stoch = (mode == DAQ_ROUND_STOCHASTIC);
    const uint64_t keys = round_keys(seed);   // what the kernels receive in the place of the seed
    const bool qg_nhwc = (Lg.kind == DAQ_LAYOUT_NHWC);
    QuantWs ws = carve_quant_ws(workspace, C, N, HW);
    ws.scheme = (int)scheme;
    const double Mtot = (double)N * (double)C * (double)HW;

    const FastDiv div_hw = make_fastdiv((uint32_t)HW);
    const int CB = (int)ceil_div(C, 64);
    const float* no_scale = nullptr;

    // Channels that fit in LDS: one read of dY serves statistics, count, decision and the per-channel copy
    // (k_chan_resident); the global copy follows in the counting kernel's copy-only form.
    // a workgroup of 512 threads x 8 or 16 load units, or 1024 x 16, holds the channel; a unit is four elements where planes are a
    // multiple of four elements long in a 16-byte aligned fp32 tensor, else one element
    const bool res_v4 = sizeof(T) == 4 && HW % 4 == 0 && ((uintptr_t)dY & 15u) == 0;
    const int64_t res_units = ceil_div((int64_t)N * HW, res_v4 ? 4 : 1);
    const bool res_small = res_units <= 8 * 512, res_mid = res_units <= 16 * 512;
    const bool resident_ok = scheme == DAQ_SCHEME_DAQ && res_units <= 16 * 1024 && Lv.plane_pitch <= kResidentMaxLds &&
                             (Lv.plane_pitch & 15) == 0 && (Lv.chan_pitch & 15) == 0;
    // (The 1024-thread form runs one workgroup per CU, whose load, count and packing phases follow each other with nothing
    // to overlap them: on 128 -> 512 at 28 x 28, batch 64, it takes 59 + 27 us against 31 + 50 + 8 us for the sweeps - level -
    // but it saves a launch, and ResNet-50's backward pass as a whole measured 1 % faster with it than without.)
    if (!given && resident_ok && (schedule == DAQ_SCHEDULE_CHANNEL_RESIDENT || schedule == DAQ_SCHEDULE_AUTO)) {
        ws.slabs = 1;   // one |g|max partial per channel
        const ResArgs ra{div_hw, make_fastdiv((uint32_t)Wo), N, C, HW, k, A, lambda, keys};
        const ClipArgs ca{k, A, lambda, s_state, s_chan, cls, stats};
        // planes without padding between rows and images hold element m at byte lead + m
        const bool res_flat = res_v4 && Lv.row_pitch == Lv.W && Lv.img_rows == Lv.H && (Lv.lead & 3) == 0 && (Lv.plane_pitch & 3) == 0 &&
                              Lv.lead + (int64_t)N * HW <= Lv.plane_pitch;
        const size_t lds = res_flat ? 0 : (size_t)Lv.plane_pitch;
#define DAQ_RES_LAUNCH(S, V, NUV, THV)                                                                               \
    if (V && res_flat) {                                                                                             \
        DAQ_LAUNCH("chan_resident", st, hipLaunchKernelGGL((k_chan_resident<T, S, V, NUV, THV, V>), dim3((unsigned)round_up(C, kXcd)), dim3(THV), 0, st, dY, cnhw_view(Lv), vq, ra, ws, ca)); \
    } else {                                                                                                         \
        auto kern = k_chan_resident<T, S, V, NUV, THV>;                                                              \
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) \
            return DAQ_ERR_HIP;                                                                                      \
        DAQ_LAUNCH("chan_resident", st, hipLaunchKernelGGL(kern, dim3((unsigned)round_up(C, kXcd)), dim3(THV), lds, st, dY, cnhw_view(Lv), vq, ra, ws, ca)); \
    }
#define DAQ_RES_SIZE(S, V) { if (res_small) DAQ_RES_LAUNCH(S, V, 8, 512) else if (res_mid) DAQ_RES_LAUNCH(S, V, 16, 512) else DAQ_RES_LAUNCH(S, V, 16, 1024) }
        if constexpr (sizeof(T) == 4) {
            if (stoch) { if (res_v4) DAQ_RES_SIZE(true, true) else DAQ_RES_SIZE(true, false) }
            else { if (res_v4) DAQ_RES_SIZE(false, true) else DAQ_RES_SIZE(false, false) }
        } else {
            if (stoch) DAQ_RES_SIZE(true, false) else DAQ_RES_SIZE(false, false)
        }
#undef DAQ_RES_SIZE
#undef DAQ_RES_LAUNCH
        // the per-channel copy, its scales, classes and clip state are complete here; the global copy follows on `st`
        if (side && stream_follows(side, st) != DAQ_OK) return DAQ_ERR_HIP;
        if (!qg_nhwc) {
            // depthwise layers: the per-tensor copy is channel-major too; its scale is folded from the channel maxima first
            DAQ_LAUNCH("fold_max", st, hipLaunchKernelGGL(k_fold_max, dim3(1), dim3(kBlock), 0, st, ws, C, s_global));
            return launch_pack("pack_qg", stoch, false, dY, Lv, s_global, 0, qg, 1u, keys, ws, ClipArgs{}, st);
        }
        const dim3 cgrid((unsigned)(CB * ws.cgroups));
#define DAQ_COPY_LAUNCH(S)                                                                                           \
    DAQ_LAUNCH("global_copy", st,                                                                                    \
               hipLaunchKernelGGL((k_count_qg<T, S, true, false, false>), cgrid, dim3(kBlock), 0, st, dY, N, C, HW, Lg.c_pitch, \
                                  div_hw, ws, no_scale, qg, keys, (const float*)s_state, s_global, EarlyVq{}, nhwc_tail(Lg)))
        if (stoch) DAQ_COPY_LAUNCH(true);
        else DAQ_COPY_LAUNCH(false);
#undef DAQ_COPY_LAUNCH
        return DAQ_OK;
    }

    // S1: statistics partials, at most 16 per channel - or the producer's: one partial per channel, read in place
    const bool vec4 = HW >= 4;   // dword-aligned 16-byte loads run at full rate; only tiny planes take the scalar path
    const unsigned sblocks = (unsigned)(round_up(C, kXcd) * ws.slabs);
    const FastDiv div_g4 = make_fastdiv((uint32_t)((HW + 3) / 4));
    if (given) {
        ws.slabs = 1;
        ws.part_max = const_cast<float*>(given->absmax);   // the consumers only read the partials
        ws.part_s1 = const_cast<double*>(given->sum);
        ws.part_s2 = const_cast<double*>(given->sumsq);
    } else if (vec4 && HW % 4 == 0)
        DAQ_LAUNCH("stats", st, hipLaunchKernelGGL((k_stats<T, true, false>), dim3(sblocks), dim3(kBlock), 0, st, dY, N, C, HW, div_g4, ws));
    else if (vec4)
        DAQ_LAUNCH("stats", st, hipLaunchKernelGGL((k_stats<T, true, true>), dim3(sblocks), dim3(kBlock), 0, st, dY, N, C, HW, div_g4, ws));
    else
        DAQ_LAUNCH("stats", st, hipLaunchKernelGGL((k_stats<T, false, false>), dim3(sblocks), dim3(kBlock), 0, st, dY, N, C, HW, div_hw, ws));

    if (scheme == DAQ_SCHEME_MCS)
        DAQ_LAUNCH("layer_stats", st, hipLaunchKernelGGL(k_layer_stats, dim3(1), dim3(kBlock), 0, st, ws, C, Mtot));

    // S2 (+ the NHWC global copy); folds the statistics itself
    const dim3 cgrid((unsigned)(CB * ws.cgroups));
    // Large gradients: the counting pass also writes the per-channel copy under a guessed class (see k_count_qg), so
    // that the third sweep over dY only touches the channels whose guess was wrong.  Small ones are bound by launch
    // latency, not by bytes, and keep the leaner counting kernel.
    // (With the producer's statistics the counting sweep is the only full read of dY: it always writes both copies.)
    const bool want_early = schedule == DAQ_SCHEDULE_EARLY_COPY || (schedule == DAQ_SCHEDULE_AUTO && (int64_t)N * C * HW >= kEarlyVqMinElems) ||
                            (given && schedule != DAQ_SCHEDULE_THREE_SWEEPS);
    const bool early = want_early && scheme == DAQ_SCHEME_DAQ && qg_nhwc && rows_vector(Lv, dY, (int)sizeof(T)) != 0 &&
                       Lv.lead + (int64_t)N * Lv.img_rows * Lv.row_pitch < ((int64_t)1 << 32);
    EarlyVq ev{};
    if (early) {
        // |g|max / sigma of M Gaussian samples is about sqrt(2 ln M), of M Laplace samples ln M / sqrt 2: halfway
        const double lnM = std::log((double)N * HW);
        ev = EarlyVq{vq, Lv.chan_pitch, (int32_t)Lv.lead, Lv.img_rows, Lv.row_pitch, Lv.W, make_fastdiv((uint32_t)Lv.W), k, A,
                     (float)(0.5 * (std::sqrt(2.0 * lnM) + lnM / std::sqrt(2.0))), Lv.W % 4 == 0 ? 1 : 0};
    }
#define DAQ_COUNT_LAUNCH(S, Q, E)                                                                                    \
    DAQ_LAUNCH("count_qg", st,                                                                                       \
               hipLaunchKernelGGL((k_count_qg<T, S, Q, true, E>), cgrid, dim3(kBlock), 0, st, dY, N, C, HW,             \
                                  qg_nhwc ? Lg.c_pitch : 0, div_hw, ws, no_scale, qg, keys, (const float*)s_state,   \
                                  s_global, ev, qg_nhwc ? nhwc_tail(Lg) : 0))
    if (early) {
        if (stoch) DAQ_COUNT_LAUNCH(true, true, true);
        else DAQ_COUNT_LAUNCH(false, true, true);
    } else if (qg_nhwc) {
        if (stoch) DAQ_COUNT_LAUNCH(true, true, false);
        else DAQ_COUNT_LAUNCH(false, true, false);
    } else {
        DAQ_COUNT_LAUNCH(false, false, false);
    }
#undef DAQ_COUNT_LAUNCH
    if (scheme == DAQ_SCHEME_MCS)
        DAQ_LAUNCH("layer_decide", st,
                   hipLaunchKernelGGL(k_layer_decide, dim3(1), dim3(kBlock), 0, st, ws, (int)cgrid.x * (kBlock / kWave), Mtot, k, A,
                                      lambda));

    // S3 + S4 + S5: discriminator, clip rule and the per-channel copy in CNHW (and the global copy for
    // depthwise layers, whose data gradient also runs channel-major)
    ClipArgs ca{k, A, lambda, s_state, s_chan, cls, stats};
    bool fused = false;
    // an NHWC global copy is complete here: the packing launch can move to the side stream.  (A channel-major global
    // copy is written by the packing launches themselves: they stay, and the side stream follows at the end.)
    hipStream_t sp = st;
    if (side && qg_nhwc) {
        if (stream_follows(side, st) != DAQ_OK) return DAQ_ERR_HIP;
        sp = side;
    }
    rc = launch_pack("pack_vq", stoch, true, dY, Lv, nullptr, 1, vq, 0u, keys, ws, ca, sp, qg_nhwc ? nullptr : qg, s_global,
                     1u, &fused, early);
    if (rc != DAQ_OK) return rc;
    if (!qg_nhwc && !fused)
        rc = launch_pack("pack_qg", stoch, false, dY, Lv, s_global, 0, qg, 1u, keys, ws, ClipArgs{}, st);
    if (rc == DAQ_OK && side && !qg_nhwc && stream_follows(side, st) != DAQ_OK) return DAQ_ERR_HIP;
    return rc;
}

}  // namespace

extern "C" daq_status daq_quantize_grad_ex(const daq_conv_desc* desc, const void* dY, float* s_state, float k, float A,
                                           float lambda, daq_round mode, uint64_t seed, const daq_quantize_opts* opts,
                                           int8_t* vq, int8_t* qg, float* s_chan, float* s_global, uint8_t* cls,
                                           float* stats, void* workspace, size_t workspace_bytes, void* stream) {
    const daq_quantize_opts def{DAQ_SCHEME_DAQ, DAQ_SCHEDULE_AUTO, 0, 0};
    const daq_quantize_opts& o = opts ? *opts : def;
    // the options arrive as plain integers: they are checked as integers, before anything treats them as enumerators
    if (o.dy_bf16 != 0 && o.dy_bf16 != 1) return DAQ_ERR_INVALID_ARG;
    if (o.scheme < DAQ_SCHEME_DAQ || o.scheme > DAQ_SCHEME_MCS || o.schedule < DAQ_SCHEDULE_AUTO || o.schedule > DAQ_SCHEDULE_CHANNEL_RESIDENT ||
        o.reserved != 0)
        return DAQ_ERR_INVALID_ARG;
    if (o.dy_bf16)
        return quantize_grad_impl<uint16_t>(desc, static_cast<const uint16_t*>(dY), s_state, k, A, lambda, mode, seed,
                                            (daq_scheme)o.scheme, (daq_schedule)o.schedule, vq, qg, s_chan, s_global, cls,
                                            stats, workspace, workspace_bytes, stream);
    return quantize_grad_impl<float>(desc, static_cast<const float*>(dY), s_state, k, A, lambda, mode, seed,
                                     (daq_scheme)o.scheme, (daq_schedule)o.schedule, vq, qg, s_chan, s_global, cls, stats,
                                     workspace, workspace_bytes, stream);
}

extern "C" daq_status daq_quantize_grad_split(const daq_conv_desc* desc, const void* dY, float* s_state, float k, float A,
                                              float lambda, daq_round mode, uint64_t seed, const daq_quantize_opts* opts,
                                              int8_t* vq, int8_t* qg, float* s_chan, float* s_global, uint8_t* cls,
                                              float* stats, void* workspace, size_t workspace_bytes, void* stream,
                                              void* side_stream) {
    const daq_quantize_opts def{DAQ_SCHEME_DAQ, DAQ_SCHEDULE_AUTO, 0, 0};
    const daq_quantize_opts& o = opts ? *opts : def;
    if (o.dy_bf16 != 0 && o.dy_bf16 != 1) return DAQ_ERR_INVALID_ARG;
    if (o.scheme < DAQ_SCHEME_DAQ || o.scheme > DAQ_SCHEME_MCS || o.schedule < DAQ_SCHEDULE_AUTO || o.schedule > DAQ_SCHEDULE_CHANNEL_RESIDENT ||
        o.reserved != 0)
        return DAQ_ERR_INVALID_ARG;
    if (o.dy_bf16)
        return quantize_grad_impl<uint16_t>(desc, static_cast<const uint16_t*>(dY), s_state, k, A, lambda, mode, seed,
                                            (daq_scheme)o.scheme, (daq_schedule)o.schedule, vq, qg, s_chan, s_global, cls,
                                            stats, workspace, workspace_bytes, stream, side_stream);
    return quantize_grad_impl<float>(desc, static_cast<const float*>(dY), s_state, k, A, lambda, mode, seed,
                                     (daq_scheme)o.scheme, (daq_schedule)o.schedule, vq, qg, s_chan, s_global, cls, stats,
                                     workspace, workspace_bytes, stream, side_stream);
}

extern "C" daq_status daq_quantize_grad_from_stats(const daq_conv_desc* desc, const void* dY, const float* ch_absmax,
                                                   const double* ch_sum, const double* ch_sumsq, float* s_state, float k,
                                                   float A, float lambda, daq_round mode, uint64_t seed,
                                                   const daq_quantize_opts* opts, int8_t* vq, int8_t* qg, float* s_chan,
                                                   float* s_global, uint8_t* cls, float* stats, void* workspace,
                                                   size_t workspace_bytes, void* stream, void* side_stream) {
    const daq_quantize_opts def{DAQ_SCHEME_DAQ, DAQ_SCHEDULE_AUTO, 0, 0};
    const daq_quantize_opts& o = opts ? *opts : def;
    if (o.dy_bf16 != 0 && o.dy_bf16 != 1) return DAQ_ERR_INVALID_ARG;
    if (o.scheme < DAQ_SCHEME_DAQ || o.scheme > DAQ_SCHEME_MCS || o.schedule < DAQ_SCHEDULE_AUTO || o.schedule > DAQ_SCHEDULE_CHANNEL_RESIDENT ||
        o.reserved != 0)
        return DAQ_ERR_INVALID_ARG;
    const ProducerStats ps{ch_absmax, ch_sum, ch_sumsq};
    if (o.dy_bf16)
        return quantize_grad_impl<uint16_t>(desc, static_cast<const uint16_t*>(dY), s_state, k, A, lambda, mode, seed,
                                            (daq_scheme)o.scheme, (daq_schedule)o.schedule, vq, qg, s_chan, s_global, cls,
                                            stats, workspace, workspace_bytes, stream, side_stream, &ps);
    return quantize_grad_impl<float>(desc, static_cast<const float*>(dY), s_state, k, A, lambda, mode, seed,
                                     (daq_scheme)o.scheme, (daq_schedule)o.schedule, vq, qg, s_chan, s_global, cls, stats,
                                     workspace, workspace_bytes, stream, side_stream, &ps);
}

extern "C" daq_status daq_quantize_grad_scheme(const daq_conv_desc* desc, const float* dY, float* s_state, float k,
                                               float A, float lambda, daq_round mode, uint64_t seed, daq_scheme scheme,
                                               int8_t* vq, int8_t* qg, float* s_chan, float* s_global, uint8_t* cls,
                                               float* stats, void* workspace, size_t workspace_bytes, void* stream) {
    const daq_quantize_opts o{(int32_t)scheme, DAQ_SCHEDULE_AUTO, 0, 0};
    return daq_quantize_grad_ex(desc, dY, s_state, k, A, lambda, mode, seed, &o, vq, qg, s_chan, s_global, cls, stats,
                                workspace, workspace_bytes, stream);
}

extern "C" daq_status daq_quantize_grad_bf16(const daq_conv_desc* desc, const uint16_t* dY_bf16, float* s_state, float k,
                                             float A, float lambda, daq_round mode, uint64_t seed, daq_scheme scheme,
                                             int8_t* vq, int8_t* qg, float* s_chan, float* s_global, uint8_t* cls,
                                             float* stats, void* workspace, size_t workspace_bytes, void* stream) {
    const daq_quantize_opts o{(int32_t)scheme, DAQ_SCHEDULE_AUTO, 1, 0};
    return daq_quantize_grad_ex(desc, dY_bf16, s_state, k, A, lambda, mode, seed, &o, vq, qg, s_chan, s_global, cls, stats,
                                workspace, workspace_bytes, stream);
}

extern "C" daq_status daq_quantize_grad(const daq_conv_desc* desc, const float* dY, float* s_state, float k, float A,
                                        float lambda, daq_round mode, uint64_t seed, int8_t* vq, int8_t* qg,
                                        float* s_chan, float* s_global, uint8_t* cls, float* stats, void* workspace,
                                        size_t workspace_bytes, void* stream) {
    return daq_quantize_grad_ex(desc, dY, s_state, k, A, lambda, mode, seed, nullptr, vq, qg, s_chan, s_global, cls, stats,
                                workspace, workspace_bytes, stream);
}

// ---------------------------------------------------------------------------------------------
// The quantizer for callers that cannot allocate: its scratch is a fixed array in device memory.
// ---------------------------------------------------------------------------------------------
// Every GPU the library runs on holds its own copy of this array, at its own address, until the process ends.
static __device__ __align__(256) unsigned char scratch[DAQ_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each device, looked up on first use

// Address of the current device's copy of the array.  In host code the array's name is only a handle for this
// lookup, never a device address: kernels, fills and copies get the pointer returned here.
daq_status static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DAQ_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return DAQ_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DAQ_OK;
}
}  // namespace

extern "C" daq_status daq_quantize_grad_noalloc(const daq_conv_desc* desc, const float* dY, float* s_state, float k, float A,
                                                float lambda, daq_round mode, uint64_t seed, int8_t* vq, int8_t* qg,
                                                float* s_chan, float* s_global, uint8_t* cls, float* stats, void* stream) {
    if (!desc_valid(desc)) return DAQ_ERR_INVALID_ARG;
    const size_t need = daq_workspace_bytes(DAQ_OP_QUANTIZE_GRAD, desc);
    if (need == 0) return DAQ_ERR_UNSUPPORTED;
    if (need > (size_t)DAQ_STATIC_SCRATCH_BYTES) return DAQ_ERR_SCRATCH_LIMIT;
    void* ws = nullptr;
    const daq_status rc = static_scratch(&ws);
    if (rc != DAQ_OK) return rc;
    // The kernels take the array through the same workspace argument as in daq_quantize_grad.  Nothing in it has to
    // start at zero: every partial result is written before it is read (no counters, no atomics).
    return daq_quantize_grad_ex(desc, dY, s_state, k, A, lambda, mode, seed, nullptr, vq, qg, s_chan, s_global, cls, stats, ws,
                                (size_t)DAQ_STATIC_SCRATCH_BYTES, stream);
}
