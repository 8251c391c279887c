// Per-channel search for the clip value that minimises the magnitude-weighted quantization error, Eq. "e":
//
//     E_c(s) = (1/M) * sum over the channel of  |g - g^(g, s)| * exp(alpha * |g|),    g^ = Q(g, s) * s / 127,
//
// evaluated on a grid of candidates s_j = |g|max_c * j / J, j = 1 .. J, for a GIVEN alpha.  This is what "solving the
// clip value" means literally in the paper's derivation; the run-time rule of Algorithm 1 (Eq. "gaus" / Eq. "fats") is
// its alpha-free closed form, so this entry point is an analysis tool beside the hot path: it lets a user see how far the
// rule's clip value is from the optimum of the objective it was derived from, on real gradients.
//
// Three launches: per-channel |g|max partials; per (channel, slab) the J partial error sums (every element's weight
// exp(alpha |g|) is computed once, in fp64, and serves all candidates); a fixed-order fold with the arg-min.
#include <algorithm>

#include "daq_internal.h"

namespace daq {

namespace {

constexpr int kBlock = 256;
constexpr int kMaxJ = 64;

struct CsWs {
    float* pmax;     // [C][S]
    double* perr;    // [C][S][kMaxJ]
    int S;           // slabs per channel
    int per_slab;    // elements of a channel one slab covers (a multiple of kBlock)
    int64_t bytes;
};

CsWs carve(void* base, int C, int64_t M) {
    CsWs w{};
    const int64_t want = std::max<int64_t>(1, 2048 / C);
    w.S = (int)std::max<int64_t>(1, std::min<int64_t>(want, ceil_div(M, 4 * kBlock)));
    w.per_slab = (int)round_up(ceil_div(M, w.S), kBlock);
    w.S = (int)ceil_div(M, w.per_slab);
    const int64_t o_err = round_up((int64_t)C * w.S * 4, 256);
    w.bytes = o_err + round_up((int64_t)C * w.S * kMaxJ * 8, 256);
    if (base) {   // a size query passes no buffer
        w.pmax = (float*)base;
        w.perr = (double*)((char*)base + o_err);
    }
    return w;
}

__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o);
    return v;
}

__global__ __launch_bounds__(kBlock) void k_cs_max(const float* __restrict__ g, int N, int C, int HW, FastDiv div_hw, CsWs ws) {
    __shared__ float l_m[kBlock / kWave];
    const int c = blockIdx.x, s = blockIdx.y, tid = threadIdx.x;
    const int M = N * HW;
    const int lo = s * ws.per_slab, hi = min(M, lo + ws.per_slab);
    float mx = 0.0f;
    for (int m = lo + tid; m < hi; m += kBlock) {
        const int n = (int)fdiv((uint32_t)m, div_hw);
        mx = fmaxf(mx, fabsf(g[((int64_t)n * C + c) * HW + (m - n * HW)]));
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_down(mx, o));
    if (tid % kWave == 0) l_m[tid / kWave] = mx;
    __syncthreads();
    if (tid == 0) ws.pmax[c * ws.S + s] = fmaxf(fmaxf(l_m[0], l_m[1]), fmaxf(l_m[2], l_m[3]));
}

__global__ __launch_bounds__(kBlock) void k_cs_err(const float* __restrict__ g, int N, int C, int HW, FastDiv div_hw, CsWs ws,
                                                   float alpha, int J) {
    __shared__ float l_inv[kMaxJ], l_step[kMaxJ];
    __shared__ double l_red[kBlock / kWave][kMaxJ];
    const int c = blockIdx.x, s = blockIdx.y, tid = threadIdx.x;
    const int M = N * HW;
    float gm = 0.0f;
    for (int i = 0; i < ws.S; ++i) gm = fmaxf(gm, ws.pmax[c * ws.S + i]);
    if (tid < kMaxJ) {
        // candidate j + 1 of J: s = |g|max * ((j + 1) / J); Eq. "suq" with its scale: codes round(clamp(x * 127/s)), g^ = code * (s/127)
        const float sj = tid < J ? gm * ((float)(tid + 1) / (float)J) : 0.0f;
        l_inv[tid] = (sj >= kTinyScale) ? 127.0f / sj : 0.0f;
        l_step[tid] = (sj >= kTinyScale) ? sj / 127.0f : 0.0f;
    }
    __syncthreads();
    double acc[kMaxJ];
#pragma unroll
    for (int j = 0; j < kMaxJ; ++j) acc[j] = 0.0;
    const int lo = s * ws.per_slab, hi = min(M, lo + ws.per_slab);
    for (int m = lo + tid; m < hi; m += kBlock) {
        const int n = (int)fdiv((uint32_t)m, div_hw);
        const float x = g[((int64_t)n * C + c) * HW + (m - n * HW)];
        const double w = exp((double)alpha * (double)fabsf(x));
#pragma unroll
        for (int j = 0; j < kMaxJ; ++j) {
            if (j < J) {   // uniform
                const float t = fminf(fmaxf(x * l_inv[j], -127.0f), 127.0f);
                const float gh = rintf(t) * l_step[j];
                acc[j] += fabs((double)x - (double)gh) * w;
            }
        }
    }
    const int wave = tid / kWave, lane = tid % kWave;
#pragma unroll
    for (int j = 0; j < kMaxJ; ++j) {
        const double v = wave_sum_d(acc[j]);
        if (lane == 0) l_red[wave][j] = v;
    }
    __syncthreads();
    if (tid < kMaxJ)
        ws.perr[((int64_t)c * ws.S + s) * kMaxJ + tid] = (l_red[0][tid] + l_red[1][tid]) + (l_red[2][tid] + l_red[3][tid]);
}

__global__ __launch_bounds__(kMaxJ) void k_cs_pick(CsWs ws, int J, double M, double* __restrict__ err, float* __restrict__ best_s,
                                                   int32_t* __restrict__ best_j) {
    __shared__ double l_e[kMaxJ];
    const int c = blockIdx.x, j = threadIdx.x;
    double e = 0.0;
    for (int s = 0; s < ws.S; ++s) e += ws.perr[((int64_t)c * ws.S + s) * kMaxJ + j];   // slab order: the same sum in every run
    e /= M;
    l_e[j] = e;
    if (err && j < J) err[(int64_t)c * J + j] = e;
    __syncthreads();
    if (j == 0) {
        int arg = 0;
        for (int i = 1; i < J; ++i)
            if (l_e[i] < l_e[arg]) arg = i;   // the smallest candidate wins a tie
        float gm = 0.0f;
        for (int i = 0; i < ws.S; ++i) gm = fmaxf(gm, ws.pmax[c * ws.S + i]);
        best_j[c] = arg + 1;
        best_s[c] = gm * ((float)(arg + 1) / (float)J);
    }
}

}  // namespace

size_t clip_search_ws_bytes(const daq_conv_desc& d) {
    return (size_t)carve(nullptr, d.Cout, (int64_t)d.N * daq_out_h(&d) * daq_out_w(&d)).bytes;
}

}  // namespace daq

using namespace daq;

extern "C" daq_status daq_clip_search(const daq_conv_desc* desc, const float* dY, float alpha, int32_t J, double* err,
                                      float* best_s, int32_t* best_j, void* workspace, size_t workspace_bytes, void* stream) {
    if (!desc_valid(desc) || !dY || !best_s || !best_j || J < 1 || J > kMaxJ || !(alpha >= 0.0f)) return DAQ_ERR_INVALID_ARG;
    if (((uintptr_t)dY & 3u) || ((uintptr_t)err & 7u)) return DAQ_ERR_INVALID_ARG;
    const size_t need = daq_workspace_bytes(DAQ_OP_CLIP_SEARCH, desc);
    if (need == 0) return DAQ_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u)) return DAQ_ERR_WORKSPACE;
    const int N = desc->N, C = desc->Cout, HW = daq_out_h(desc) * daq_out_w(desc);
    const int64_t M = (int64_t)N * HW;
    if (M * C >= ((int64_t)1 << 31) || C > 65535) return DAQ_ERR_UNSUPPORTED;
    const CsWs ws = carve(workspace, C, M);
    hipStream_t st = (hipStream_t)stream;
    const FastDiv div_hw = make_fastdiv((uint32_t)HW);
    const dim3 grid((unsigned)C, (unsigned)ws.S);
    DAQ_LAUNCH("clip_search_max", st, hipLaunchKernelGGL(k_cs_max, grid, dim3(kBlock), 0, st, dY, N, C, HW, div_hw, ws));
    DAQ_LAUNCH("clip_search_err", st, hipLaunchKernelGGL(k_cs_err, grid, dim3(kBlock), 0, st, dY, N, C, HW, div_hw, ws, alpha, (int)J));
    DAQ_LAUNCH("clip_search_pick", st,
               hipLaunchKernelGGL(k_cs_pick, dim3((unsigned)C), dim3(kMaxJ), 0, st, ws, (int)J, (double)M, err, best_s, best_j));
    return DAQ_OK;
}
