// Last stage of a K-split filter gradient as a ROLE that workgroups of another kernel can take on.
//
// The K-split kernels of conv_mfma_dw32.hip leave `splits` int32 partial tiles per output tile; summing them and
// applying the de-quantization  dW = acc * (s_x/127) * (s_chan[co]/127)  (vectorized de-quantization formula,
// Algorithm 1) is a few microseconds of plain loads.  As a launch of its own it costs a dependent-launch gap on
// top; when the caller asks for both gradients of a layer in one call, the data-gradient kernel - which does not
// depend on the filter gradient - is launched with extra workgroups that do this sum instead.
//
// Those workgroups inherit the host kernel's registers and LDS, so few of them fit on a CU and each costs a
// dispatch slot the host kernel's own tiles could use: the role pays off where every workgroup of it has many
// partial tiles to sum (early layers: few output tiles, many K splits) and is not used otherwise
// (dw_tail_worthwhile; measured on the ResNet-50 shapes).
#pragma once

#include "daq_internal.h"

namespace daq {

struct DwTail {
    const int32_t* part;   // [tile][split][wave tile][slot][lane]
    int blocks;            // workgroups of this role, one per group of 64 consecutive (slot, lane) results; 0 = no role
    int splits, tiles_n, wm_n, wn_n, Cout, Cin;
    int taps;              // 9: 32 x 32 x 9 wave tiles (3 x 3 filters); 1: 64 x 64 wave tiles (1 x 1 filters)
    const float* s_x;
    const float* s_chan;
    float* dW;
    int32_t* acc_out;
    int bf16;              // dW is bfloat16 storage
};

// Whether the role should replace the reduction launch: one workgroup per entry, each with more than 32 splits.
inline bool dw_tail_worthwhile(int entries, int splits) { return splits > 32 && entries <= 4096; }

// Entry e, lane -> element of dW (or -1 outside the tensor) and its output channel.
__device__ __forceinline__ int64_t dw_tail_element(const DwTail& t, int e, int lane, int& co) {
    const int per_wave = t.taps == 9 ? 9 * 16 : 64;      // slots of one wave tile
    const int wtiles = t.wm_n * t.wn_n;
    const int slot = e % per_wave;
    const int wt = (e / per_wave) % wtiles;
    const int tile = e / (per_wave * wtiles);
    const int wm = wt / t.wn_n, wn = wt % t.wn_n;
    const int tm = tile / t.tiles_n, tn = tile % t.tiles_n;
    const int r = slot % 16;
    int ci;
    int64_t off;
    if (t.taps == 9) {
        // register r of tap slot/16: row (co) 8*(r/4) + 4*(lane/32) + r%4, column (ci) lane%32
        co = (tm * t.wm_n + wm) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        ci = (tn * t.wn_n + wn) * 32 + (lane & 31);
        off = ((int64_t)co * t.Cin + ci) * 9 + slot / 16;
    } else {
        co = (tm * t.wm_n + wm) * 64 + 32 * (slot / 32) + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        ci = (tn * t.wn_n + wn) * 64 + 32 * ((slot / 16) % 2) + (lane & 31);
        off = (int64_t)co * t.Cin + ci;
    }
    return (co < t.Cout && ci < t.Cin) ? off : -1;
}

// Partial sums of entry e start here; consecutive splits are `stride` ints apart.
__device__ __forceinline__ const int32_t* dw_tail_source(const DwTail& t, int e, int lane, int64_t& stride) {
    const int per_tile = (t.taps == 9 ? 9 * 16 : 64) * t.wm_n * t.wn_n;   // entries of one output tile
    stride = (int64_t)per_tile * kWave;
    const int tile = e / per_tile;
    return t.part + (int64_t)tile * t.splits * stride + (int64_t)(e - tile * per_tile) * kWave + lane;
}

// Workgroup `e` of the role (one entry); `scratch` is at least (blockDim.x / 64) * 64 ints of LDS.  Every wave of
// the workgroup must call it (it contains a barrier); the waves take the splits round robin.
__device__ __forceinline__ void dw_reduce_role(const DwTail& t, int e, int32_t* scratch) {
    const int lane = threadIdx.x % kWave, grp = threadIdx.x / kWave, nw = blockDim.x / kWave;
    int64_t stride;
    const int32_t* src = dw_tail_source(t, e, lane, stride);
    int32_t a = 0;
    int s = grp;
    for (; s + 7 * nw < t.splits; s += 8 * nw) {
        int32_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[(int64_t)(s + nw * u) * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) a += v[u];
    }
    for (; s < t.splits; s += nw) a += src[(int64_t)s * stride];
    scratch[grp * kWave + lane] = a;
    __syncthreads();
    if (grp != 0) return;
    a = 0;
    for (int w = 0; w < nw; ++w) a += scratch[w * kWave + lane];
    int co;
    const int64_t off = dw_tail_element(t, e, lane, co);
    if (off < 0) return;
    store_result(t.dW, off, (float)a * ((*t.s_x / 127.0f) * (t.s_chan[co] / 127.0f)), t.bf16);
    if (t.acc_out) t.acc_out[off] = a;
}

}  // namespace daq
