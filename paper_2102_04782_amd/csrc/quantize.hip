// Gradient Vectorized Quantization on gfx950: channel statistics, discriminator + clip solve,
// and the int8 packing kernels (Algorithm 1, per-channel loop and the two quantizations), plus
// the per-tensor quantization of X and W used by the forward pass.
//
// All kernels here are bandwidth bound.  Float reductions use fixed trees and a fixed-order
// second stage (no float atomics), so results do not depend on scheduling.  Compile with
// -ffp-contract=off: the rounding of every fp32/fp64 expression below is part of the contract.
#include <algorithm>

#include "daq_internal.h"

namespace daq {

namespace {

constexpr int kBlock = 256;
constexpr int kStatsElems = 4096;  // elements swept by one statistics workgroup (16 per thread, all loads in flight)

// ---------------------------------------------------------------------------------------------
// workspace carving
// ---------------------------------------------------------------------------------------------
struct QuantWs {
    uint32_t* gmax_bits;  // [1]   bit pattern of max_c |g|max (non-negative floats order like uints)
    float* gmax;          // [C]
    float* mean;          // [C]
    float* sigma;         // [C]
    float* part_max;      // [C][chunks]
    double* part_s1;      // [C][chunks]
    double* part_s2;      // [C][chunks]
    uint32_t* part_cnt;   // [C][slots]  #{|g| > sigma} per (image, 64-pixel tile)
    int chunks, slots;
    int64_t total_bytes;
};

QuantWs carve_quant_ws(void* base, int C, int N, int HW) {
    QuantWs w{};
    char* p = (char*)base;
    const int64_t M = (int64_t)N * HW;
    w.chunks = (int)ceil_div(M, kStatsElems);
    w.slots = N * (int)ceil_div(HW, kWave);
    w.gmax_bits = (uint32_t*)p;
    p += 256;
    w.gmax = (float*)p;
    w.mean = w.gmax + C;
    w.sigma = w.mean + C;
    p += round_up((int64_t)3 * C * 4, 256);
    w.part_s1 = (double*)p;
    w.part_s2 = w.part_s1 + (int64_t)C * w.chunks;
    p += round_up((int64_t)2 * C * w.chunks * 8, 256);
    w.part_max = (float*)p;
    p += round_up((int64_t)C * w.chunks * 4, 256);
    w.part_cnt = (uint32_t*)p;
    p += round_up((int64_t)C * w.slots * 4, 256);
    w.total_bytes = p - (char*)base;
    return w;
}

// ---------------------------------------------------------------------------------------------
// device helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// 24-bit uniform in [0,1) keyed by (seed, tensor, element index): SplitMix64 output function of a counter.
__device__ __forceinline__ float uniform24(uint64_t seed, uint32_t tensor, uint64_t idx) {
    const uint64_t ctr = seed + 0x9E3779B97F4A7C15ull * (idx + 1) + 0xD1B54A32D192ED03ull * (uint64_t)tensor;
    return (float)(uint32_t)(mix64(ctr) >> 40) * 5.9604644775390625e-08f;
}

// 127/s, or 0 when the scale is treated as zero (then every code is 0).
__device__ __forceinline__ float inv_scale(float s) { return (s >= kTinyScale) ? 127.0f / s : 0.0f; }

// Eq. "suq" in code space: round(clamp(x*inv, -127, 127)).
template <bool STOCH>
__device__ __forceinline__ int quant_code(float x, float inv, uint64_t seed, uint32_t tensor, uint64_t idx) {
    float t = x * inv;
    t = fminf(fmaxf(t, -127.0f), 127.0f);
    if (STOCH) {
        const float f = floorf(t);
        const float frac = t - f;
        const float u = uniform24(seed, tensor, idx);
        return (int)(f + (frac > u ? 1.0f : 0.0f));
    }
    return (int)rintf(t);
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
// S1: per-channel |g|max, sum, sum of squares.  Workgroup (c, j) sweeps elements
// [j*4096, (j+1)*4096) of channel c's flattened (n, h*w) axis with every load issued up front,
// and stores one partial.  k_stats_final reduces a channel's partials with a fixed tree.
// Channel c runs on XCD c % 8 in every pass over dY.
// ---------------------------------------------------------------------------------------------
template <bool VEC4>
__global__ __launch_bounds__(kBlock) void k_stats(const float* __restrict__ g, int N, int C, int HW, QuantWs ws) {
    const int b = blockIdx.x;
    const int xcd = b % kXcd, q = b / kXcd;
    const int c = (q / ws.chunks) * kXcd + xcd;
    const int j = q % ws.chunks;
    if (b == 0 && threadIdx.x == 0) *ws.gmax_bits = 0u;  // consumed by k_stats_final, a later launch
    if (c >= C) return;
    const int M = N * HW;
    const int m0 = j * kStatsElems;
    const int tid = threadIdx.x;

    float mx = 0.0f;
    double s1 = 0.0, s2 = 0.0;
    if (VEC4) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int m = m0 + 4 * (tid + u * kBlock);
            const bool ok = m < M;
            const int mc = ok ? m : 0;
            const int n = mc / HW, i = mc - n * HW;
            const uint4 raw = ld16_or_zero(g + ((int64_t)n * C + c) * HW + i, ok);
            v[u] = make_float4(__uint_as_float(raw.x), __uint_as_float(raw.y), __uint_as_float(raw.z),
                               __uint_as_float(raw.w));
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            mx = fmaxf(mx, fmaxf(fmaxf(fabsf(v[u].x), fabsf(v[u].y)), fmaxf(fabsf(v[u].z), fabsf(v[u].w))));
            const double a = v[u].x, bq = v[u].y, cq = v[u].z, d = v[u].w;
            s1 += a; s1 += bq; s1 += cq; s1 += d;
            s2 += a * a; s2 += bq * bq; s2 += cq * cq; s2 += d * d;
        }
    } else {
        float v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int m = m0 + tid + u * kBlock;
            const bool ok = m < M;
            const int mc = ok ? m : 0;
            const int n = mc / HW, i = mc - n * HW;
            v[u] = ldf_or_zero(g + ((int64_t)n * C + c) * HW + i, ok);
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            mx = fmaxf(mx, fabsf(v[u]));
            const double a = v[u];
            s1 += a;
            s2 += a * a;
        }
    }
    block_reduce(mx, s1, s2);
    if (tid == 0) {
        const int64_t slot = (int64_t)c * ws.chunks + j;
        ws.part_max[slot] = mx;
        ws.part_s1[slot] = s1;
        ws.part_s2[slot] = s2;
    }
}

// One workgroup per channel: partials -> |g|max, mean, sigma (population std, fp64, rounded once).
__global__ __launch_bounds__(kBlock) void k_stats_final(int N, int C, int HW, QuantWs ws) {
    const int c = blockIdx.x;
    float mx = 0.0f;
    double s1 = 0.0, s2 = 0.0;
    for (int j = threadIdx.x; j < ws.chunks; j += kBlock) {
        const int64_t slot = (int64_t)c * ws.chunks + j;
        mx = fmaxf(mx, ws.part_max[slot]);
        s1 += ws.part_s1[slot];
        s2 += ws.part_s2[slot];
    }
    block_reduce(mx, s1, s2);
    if (threadIdx.x == 0) {
        const double Md = (double)N * (double)HW;
        const double mu = s1 / Md;
        double var = s2 / Md - mu * mu;
        if (var < 0.0) var = 0.0;
        ws.gmax[c] = mx;
        ws.mean[c] = (float)mu;
        ws.sigma[c] = (float)sqrt(var);
        atomicMax(ws.gmax_bits, __float_as_uint(mx));
    }
}

// ---------------------------------------------------------------------------------------------
// S2 (+ the global copy of S5): tail-mass count per channel, fused with the globally quantized
// NHWC copy.  A workgroup owns 64 pixels of one image and 64 channels; wave w walks channels
// 16w..16w+15 with lane = pixel, so every load is a 256-byte run of one channel and the lane's 16
// codes are 16 contiguous bytes of the NHWC output.  Counts are wave ballots, stored per
// (channel, image, pixel tile) and summed by k_clip_final: no atomics anywhere.
// ---------------------------------------------------------------------------------------------
struct ClipArgs {
    float k, A, lambda;
    float* s_state;
    float* s_chan;
    float* s_global;
    uint8_t* cls;
    float* stats;
};

template <bool STOCH, bool WRITE_QG, bool COUNT>
__global__ __launch_bounds__(kBlock) void k_count_qg(const float* __restrict__ g, int N, int C, int HW, int c_pitch,
                                                     int ptiles, QuantWs ws, const float* __restrict__ scale_ptr,
                                                     int8_t* __restrict__ qg, uint64_t seed) {
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    int b = blockIdx.x;
    const int pt = b % ptiles; b /= ptiles;
    const int n = b % N;
    const int cb = b / N;
    const int c0 = cb * 64 + 16 * wave;
    const int px = pt * kWave + lane;
    const bool vpx = px < HW;

    // scale of the global copy: max_c |g|max from the statistics pass, or an explicit per-tensor scale
    float sg = 0.0f;
    if (WRITE_QG) {
        sg = scale_ptr ? *scale_ptr : __uint_as_float(*ws.gmax_bits);
        if (!(sg >= kTinyScale)) sg = 0.0f;
    }
    const float inv = inv_scale(sg);

    const float* gp = g + ((int64_t)n * C + c0) * HW + px;
    float x[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = ldf_or_zero(gp + (int64_t)i * HW, vpx && c0 + i < C);

    uint32_t mycnt = 0;
    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int c = c0 + i;
        if (COUNT) {
            const float sig = (c < C) ? ws.sigma[c] : 0.0f;
            const unsigned long long bal = __ballot(vpx && c < C && fabsf(x[i]) > sig);
            if (lane == i) mycnt = (uint32_t)__popcll(bal);
        }
        if (WRITE_QG) {
            const uint64_t idx = (uint64_t)(((int64_t)n * C + c) * HW + px);
            const int code = quant_code<STOCH>(x[i], inv, seed, 1u, idx);
            w[i >> 2] |= ((uint32_t)code & 0xFFu) << (8 * (i & 3));
        }
    }
    if (WRITE_QG && vpx && c0 < c_pitch)
        *reinterpret_cast<uint4*>(qg + ((int64_t)n * HW + px) * c_pitch + c0) = make_uint4(w[0], w[1], w[2], w[3]);
    if (COUNT && lane < 16 && c0 + lane < C)
        ws.part_cnt[(int64_t)(c0 + lane) * ws.slots + n * ptiles + pt] = mycnt;
}

// S2 (sum of the partial counts) + S3 discriminator + S4 clip rule, one workgroup per channel.
__global__ __launch_bounds__(kBlock) void k_clip_final(int N, int C, int HW, QuantWs ws, ClipArgs ca) {
    const int c = blockIdx.x;
    uint32_t cnt = 0;
    for (int j = threadIdx.x; j < ws.slots; j += kBlock) cnt += ws.part_cnt[(int64_t)c * ws.slots + j];
    cnt = wave_sum_u32(cnt);
    __shared__ uint32_t l_cnt[kBlock / kWave];
    if (threadIdx.x % kWave == 0) l_cnt[threadIdx.x / kWave] = cnt;
    __syncthreads();
    if (threadIdx.x != 0) return;
    for (int w = 1; w < kBlock / kWave; ++w) cnt += l_cnt[w];

    float sg = __uint_as_float(*ws.gmax_bits);
    if (!(sg >= kTinyScale)) sg = 0.0f;
    if (c == 0) *ca.s_global = sg;
    const double Md = (double)N * (double)HW;
    const int klass = ((double)cnt > (double)ca.lambda * Md) ? DAQ_CLASS_GAUSS : DAQ_CLASS_INVT;
    const float gm = ws.gmax[c];
    float s = gm;
    if (klass == DAQ_CLASS_INVT) {
        float p = ca.s_state[c];
        if (!(p > 0.0f)) p = gm;
        s = (float)((1.0 - (double)ca.k * (double)ca.A) * (double)p + (double)ca.A * (double)gm);
        if (!(s > 0.0f)) s = gm;
    }
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

// ---------------------------------------------------------------------------------------------
// S5, channel-major copy: fp32 NCHW -> int8 CNHW (the dimension transformation G -> G', X -> X').
// Output driven: each thread produces 16 aligned bytes of the destination plane, including the
// zero bytes that serve as convolution padding, so stores are fully coalesced, every byte of the
// buffer is written exactly once and all 16 loads of a thread are in flight together.
// ---------------------------------------------------------------------------------------------
template <bool STOCH>
__global__ __launch_bounds__(kBlock) void k_pack_cnhw(const float* __restrict__ src, CnhwView L,
                                                      const float* __restrict__ scale, int per_channel,
                                                      int8_t* __restrict__ dst, uint64_t seed, uint32_t tensor,
                                                      int per_chan) {
    const int b = blockIdx.x;
    const int xcd = b % kXcd, q = b / kXcd;
    const int c = (q / per_chan) * kXcd + xcd;  // channel c runs on XCD c % 8
    const int jb = q % per_chan;                // block of 16-byte units along the flattened axis
    const int phase = blockIdx.z;
    if (c >= L.C) return;
    const int64_t j = (int64_t)jb * kBlock + threadIdx.x;  // 16-byte unit inside the plane
    if (16 * j >= L.plane_pitch) return;
    const int ph = phase / L.phases_w, pw = phase % L.phases_w;
    const float inv = inv_scale(per_channel ? scale[c] : scale[0]);

    const int slot = L.img_rows * L.row_pitch;
    int64_t o = 16 * j - L.lead;
    int n = 0, r = 0, col = 0;
    if (o > 0) {
        n = (int)(o / slot);
        const int rem = (int)(o - (int64_t)n * slot);
        r = rem / L.row_pitch;
        col = rem - r * L.row_pitch;
    }
    float x[16];
    int64_t idx[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        x[i] = 0.0f;
        idx[i] = -1;
        if (o + i >= 0) {
            const int h = r * L.phases_h + ph - L.org_h;
            const int w = col * L.phases_w + pw - L.org_w;
            const bool ok = n < L.N && h >= 0 && h < L.H && w >= 0 && w < L.W;
            idx[i] = ok ? (((int64_t)n * L.C + c) * L.H + h) * L.W + w : -1;
            x[i] = ldf_or_zero(src + idx[i], ok);
            if (++col == L.row_pitch) {
                col = 0;
                if (++r == L.img_rows) { r = 0; ++n; }
            }
        }
    }
    uint32_t w4[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int code = (idx[i] >= 0) ? quant_code<STOCH>(x[i], inv, seed, tensor, (uint64_t)idx[i]) : 0;
        w4[i >> 2] |= ((uint32_t)code & 0xFFu) << (8 * (i & 3));
    }
    *reinterpret_cast<uint4*>(dst + (int64_t)c * L.chan_pitch + (int64_t)phase * L.plane_pitch + 16 * j) =
        make_uint4(w4[0], w4[1], w4[2], w4[3]);
}

// ---------------------------------------------------------------------------------------------
// per-tensor helpers for the forward pass
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_absmax(const float* __restrict__ x, int64_t n, uint32_t* bits) {
    float m = 0.0f;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock)
        m = fmaxf(m, fabsf(x[i]));
    m = wave_max(m);
    if (threadIdx.x % kWave == 0) atomicMax(bits, __float_as_uint(m));
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
    const int8_t code = (int8_t)quant_code<false>(W[i], inv, 0, 0, 0);
    out[L.off_plain + i] = code;
    out[L.off_fwd + ((int64_t)tap * Cout + co) * L.cig_pitch + cl] = code;
    out[L.off_bwd + ((int64_t)tap * Cin + ci) * L.cog_pitch + col] = code;
}

// grid of k_pack_cnhw: x enumerates (channel, block of 16-byte units) with the channel's XCD in the low bits,
// z the stride phase
int pack_per_chan(const daq_layout& L) { return (int)ceil_div(L.plane_pitch / 16, kBlock); }
dim3 pack_grid(const daq_layout& L) {
    return dim3((unsigned)(round_up(L.C, kXcd) * pack_per_chan(L)), 1u, (unsigned)(L.phases_h * L.phases_w));
}

}  // namespace

size_t quantize_grad_ws_bytes(const daq_conv_desc& d) {
    return (size_t)carve_quant_ws(nullptr, d.Cout, d.N, daq_out_h(&d) * daq_out_w(&d)).total_bytes;
}

size_t fwd_quant_ws_bytes(const daq_conv_desc&) { return 256; }

// ---------------------------------------------------------------------------------------------
// forward-side quantization of X (two layouts) and W (packed)
// ---------------------------------------------------------------------------------------------
daq_status quantize_activation(const daq_conv_desc& d, const float* X, int8_t* qx_nhwc, int8_t* qx_cnhw, float* s_x,
                               void* wsp, hipStream_t st) {
    uint32_t* bits = (uint32_t*)wsp;
    const int64_t n = (int64_t)d.N * d.Cin * d.Hin * d.Win;
    DAQ_LAUNCH("fill", st, hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, st, bits, (int64_t)1, 0u));
    const int blocks = (int)std::min<int64_t>(ceil_div(n, kBlock * 8), 4096);
    DAQ_LAUNCH("absmax", st, hipLaunchKernelGGL(k_absmax, dim3(blocks), dim3(kBlock), 0, st, X, n, bits));
    DAQ_LAUNCH("scale", st, hipLaunchKernelGGL(k_scale_from_bits, dim3(1), dim3(1), 0, st, bits, s_x));

    daq_layout Ln, Lc;
    if (daq_layout_qx_nhwc(&d, &Ln) != DAQ_OK || daq_layout_qx_cnhw(&d, &Lc) != DAQ_OK) return DAQ_ERR_INVALID_ARG;
    const int HW = d.Hin * d.Win;
    const int ptiles = (int)ceil_div(HW, kWave);
    const int CB = (int)ceil_div(d.Cin, 64);
    QuantWs none{};
    DAQ_LAUNCH("quant_nhwc", st,
               hipLaunchKernelGGL((k_count_qg<false, true, false>), dim3(CB * d.N * ptiles), dim3(kBlock), 0, st, X,
                                  d.N, d.Cin, HW, Ln.c_pitch, ptiles, none, (const float*)s_x, qx_nhwc, (uint64_t)0));
    DAQ_LAUNCH("pack_cnhw", st,
               hipLaunchKernelGGL((k_pack_cnhw<false>), pack_grid(Lc), dim3(kBlock), 0, st, X, cnhw_view(Lc),
                                  (const float*)s_x, 0, qx_cnhw, (uint64_t)0, 0u, pack_per_chan(Lc)));
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
    const int blocks = (int)std::min<int64_t>(ceil_div(n, kBlock * 8), 4096);
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
extern "C" daq_status daq_quantize_grad(const daq_conv_desc* desc, const float* dY, float* s_state, float k, float A,
                                        float lambda, daq_round mode, uint64_t seed, int8_t* vq, int8_t* qg,
                                        float* s_chan, float* s_global, uint8_t* cls, float* stats, void* workspace,
                                        size_t workspace_bytes, void* stream) {
    if (!desc_valid(desc) || !dY || !s_state || !vq || !qg || !s_chan || !s_global || !cls)
        return DAQ_ERR_INVALID_ARG;
    if (mode != DAQ_ROUND_NEAREST && mode != DAQ_ROUND_STOCHASTIC) return DAQ_ERR_INVALID_ARG;
    daq_layout Lv, Lg;
    daq_status rc = daq_layout_vq(desc, &Lv);
    if (rc != DAQ_OK) return rc;
    rc = daq_layout_qg(desc, &Lg);
    if (rc != DAQ_OK) return rc;
    const size_t need = daq_workspace_bytes(DAQ_OP_QUANTIZE_GRAD, desc);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u)) return DAQ_ERR_WORKSPACE;

    hipStream_t st = (hipStream_t)stream;
    const int N = desc->N, C = desc->Cout, Ho = daq_out_h(desc), Wo = daq_out_w(desc);
    const int HW = Ho * Wo, M = N * HW;
    const bool stoch = (mode == DAQ_ROUND_STOCHASTIC);
    const bool qg_nhwc = (Lg.kind == DAQ_LAYOUT_NHWC);
    QuantWs ws = carve_quant_ws(workspace, C, N, HW);
    (void)M;

    // S1: partial statistics, then one workgroup per channel folds them
    const bool vec4 = (HW % 4 == 0) && (((uintptr_t)dY & 15u) == 0);
    const unsigned sblocks = (unsigned)(round_up(C, kXcd) * ws.chunks);
    if (vec4)
        DAQ_LAUNCH("stats", st, hipLaunchKernelGGL((k_stats<true>), dim3(sblocks), dim3(kBlock), 0, st, dY, N, C, HW, ws));
    else
        DAQ_LAUNCH("stats", st, hipLaunchKernelGGL((k_stats<false>), dim3(sblocks), dim3(kBlock), 0, st, dY, N, C, HW, ws));
    DAQ_LAUNCH("stats_final", st, hipLaunchKernelGGL(k_stats_final, dim3(C), dim3(kBlock), 0, st, N, C, HW, ws));

    // S2 (+ the NHWC global copy), then S3 + S4
    ClipArgs ca{k, A, lambda, s_state, s_chan, s_global, cls, stats};
    const int ptiles = (int)ceil_div(HW, kWave);
    const int CB = (int)ceil_div(C, 64);
    const dim3 cgrid((unsigned)(CB * N * ptiles));
    const float* no_scale = nullptr;
#define DAQ_COUNT_LAUNCH(S, Q)                                                                                       \
    DAQ_LAUNCH("count_qg", st,                                                                                       \
               hipLaunchKernelGGL((k_count_qg<S, Q, true>), cgrid, dim3(kBlock), 0, st, dY, N, C, HW,                \
                                  qg_nhwc ? Lg.c_pitch : 0, ptiles, ws, no_scale, qg, seed))
    if (qg_nhwc) {
        if (stoch) DAQ_COUNT_LAUNCH(true, true);
        else DAQ_COUNT_LAUNCH(false, true);
    } else {
        DAQ_COUNT_LAUNCH(false, false);
    }
#undef DAQ_COUNT_LAUNCH
    DAQ_LAUNCH("clip_final", st, hipLaunchKernelGGL(k_clip_final, dim3(C), dim3(kBlock), 0, st, N, C, HW, ws, ca));

    // S5: per-channel copy (and the global copy for depthwise layers) in CNHW
    const CnhwView V = cnhw_view(Lv);
    const dim3 pgrid = pack_grid(Lv);
    if (stoch)
        DAQ_LAUNCH("pack_vq", st,
                   hipLaunchKernelGGL((k_pack_cnhw<true>), pgrid, dim3(kBlock), 0, st, dY, V, (const float*)s_chan, 1,
                                      vq, seed, 0u, pack_per_chan(Lv)));
    else
        DAQ_LAUNCH("pack_vq", st,
                   hipLaunchKernelGGL((k_pack_cnhw<false>), pgrid, dim3(kBlock), 0, st, dY, V, (const float*)s_chan,
                                      1, vq, seed, 0u, pack_per_chan(Lv)));
    if (!qg_nhwc) {
        if (stoch)
            DAQ_LAUNCH("pack_qg", st,
                       hipLaunchKernelGGL((k_pack_cnhw<true>), pgrid, dim3(kBlock), 0, st, dY, V,
                                          (const float*)s_global, 0, qg, seed, 1u, pack_per_chan(Lv)));
        else
            DAQ_LAUNCH("pack_qg", st,
                       hipLaunchKernelGGL((k_pack_cnhw<false>), pgrid, dim3(kBlock), 0, st, dY, V,
                                          (const float*)s_global, 0, qg, seed, 1u, pack_per_chan(Lv)));
    }
    return DAQ_OK;
}
