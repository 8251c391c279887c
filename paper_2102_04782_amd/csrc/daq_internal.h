// Internal declarations shared by the translation units of libdaq.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "daq.h"

namespace daq {

constexpr int kWave = 64;            // CDNA wavefront width
constexpr int kXcd = 8;              // accelerator complex dies; workgroup i is dispatched to XCD i % 8
constexpr float kTinyScale = 7.888609052210118e-31f;  // 2^-100: below this a scale is reported as 0
// fp32 results of at least this many bytes leave through streaming (nontemporal) stores: written back as they are
// produced instead of at the end of the kernel, and without evicting the int8 operands the next kernels read.
// Smaller results stay in the write-back caches, which is faster for them (measured: 12.8 MB slower, 25.7 MB faster).
constexpr int64_t kStreamBytes = (int64_t)24 << 20;
constexpr int kKAlign = 256;         // the flattened (n,h,w) axis of a CNHW buffer is padded to this many bytes

inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

bool desc_valid(const daq_conv_desc* d);
inline bool is_depthwise(const daq_conv_desc& d) { return d.groups > 1 && d.groups == d.Cin && d.groups == d.Cout; }

// ---- profiling hooks (prof.hip) ------------------------------------------------------------
bool prof_active();
void prof_push(const char* name, hipStream_t s);  // records the start event
void prof_pop(hipStream_t s);                     // records the stop event

// Launch helper: brackets the launch with profiling events when enabled and maps launch errors.
#define DAQ_LAUNCH(name, stream, ...)                          \
    do {                                                       \
        if (::daq::prof_active()) ::daq::prof_push(name, stream); \
        __VA_ARGS__;                                           \
        if (::daq::prof_active()) ::daq::prof_pop(stream);     \
        if (hipGetLastError() != hipSuccess) return DAQ_ERR_HIP; \
    } while (0)

// ---- predicated loads without control flow ------------------------------------------------
// A load guarded by an `if` becomes an exec-masked branch with a full memory wait at its join, and a
// select applied to the loaded value makes the compiler wait right behind the load; either way a
// software pipeline is serialised.  These helpers always issue the load and redirect a false
// predicate to 64 bytes of zeros in device memory, so nothing depends on the value until it is used.
static __device__ uint4 g_zero64[4];  // zero-initialised, never written (kept non-const so it shares the global address space)
__device__ __forceinline__ uint4 ld16_or_zero(const void* p, bool ok) {
    return *reinterpret_cast<const uint4*>(ok ? p : (const void*)g_zero64);
}
__device__ __forceinline__ float ldf_or_zero(const float* p, bool ok) {
    return *(ok ? p : reinterpret_cast<const float*>(g_zero64));
}

// ---- results that are fp32 or, on request, bfloat16 -------------------------------------------
// fp32 -> bfloat16 bits, round to nearest even (finite inputs)
__device__ __forceinline__ uint32_t bf16_bits(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
// Element `off` of a result tensor whose storage is fp32, or bfloat16 when `bf16` is set (uniform).
__device__ __forceinline__ void store_result(float* base, int64_t off, float v, int bf16) {
    if (bf16) reinterpret_cast<uint16_t*>(base)[off] = (uint16_t)bf16_bits(v);
    else base[off] = v;
}
// Four consecutive results starting at element `off`, a multiple of four: one 16-byte store, or one 8-byte store of
// four bfloat16; `nt` asks for a streaming store.
typedef float daq_v4f __attribute__((ext_vector_type(4)));
typedef uint32_t daq_v2u __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void store_result4(float* base, int64_t off, float a, float b, float c, float d, int bf16, int nt) {
    if (bf16) {
        const daq_v2u w = {bf16_bits(a) | (bf16_bits(b) << 16), bf16_bits(c) | (bf16_bits(d) << 16)};
        daq_v2u* z = reinterpret_cast<daq_v2u*>(reinterpret_cast<uint16_t*>(base) + off);
        if (nt) __builtin_nontemporal_store(w, z);
        else *z = w;
    } else {
        const daq_v4f w = {a, b, c, d};
        daq_v4f* z = reinterpret_cast<daq_v4f*>(base + off);
        if (nt) __builtin_nontemporal_store(w, z);
        else *z = w;
    }
}

// ---- division by a launch-invariant divisor ---------------------------------------------------
// Exact unsigned division by an invariant divisor (Granlund-Montgomery round-up multiplier).
struct FastDiv {
    uint32_t mul;
    int32_t shift;
    int32_t one;
};
inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f{};
    f.one = (d == 1);
    int L = 0;
    while (((uint64_t)1 << L) < d) ++L;
    f.shift = L > 0 ? L - 1 : 0;
    f.mul = (uint32_t)((((uint64_t)1 << 32) * (((uint64_t)1 << L) - d)) / d + 1);
    return f;
}
__device__ __forceinline__ uint32_t fdiv(uint32_t x, const FastDiv& f) {
    const uint32_t t = __umulhi(x, f.mul);
    const uint32_t q = (t + ((x - t) >> 1)) >> f.shift;
    return f.one ? x : q;   // a select, not a branch: branches here split the prologues that call this many times
}

// ---- device-side view of an int8 layout ----------------------------------------------------
struct CnhwView {
    int64_t chan_pitch, plane_pitch, lead;
    int32_t img_rows, row_pitch;
    int32_t phases_h, phases_w, org_h, org_w;
    int32_t C, N, H, W;
    __host__ __device__ int64_t offset(int n, int c, int h, int w) const {
        const int hh = h + org_h, ww = w + org_w;
        const int ph = hh % phases_h, pw = ww % phases_w;
        return (int64_t)c * chan_pitch + (int64_t)(ph * phases_w + pw) * plane_pitch + lead +
               ((int64_t)n * img_rows + hh / phases_h) * row_pitch + ww / phases_w;
    }
};

struct NhwcView {
    int32_t c_pitch, C, N, H, W;
    __host__ __device__ int64_t offset(int n, int c, int h, int w) const {
        return (((int64_t)n * H + h) * W + w) * c_pitch + c;
    }
};

inline CnhwView cnhw_view(const daq_layout& L) {
    return CnhwView{L.chan_pitch, L.plane_pitch, L.lead, L.img_rows, L.row_pitch, L.phases_h, L.phases_w,
                    L.org_h, L.org_w, L.C, L.N, L.H, L.W};
}
inline NhwcView nhwc_view(const daq_layout& L) { return NhwcView{L.c_pitch, L.C, L.N, L.H, L.W}; }

// ---- kernels behind the entry points (one translation unit each) -----------------------------
// quantize.hip
size_t quantize_grad_ws_bytes(const daq_conv_desc& d);
size_t fwd_quant_ws_bytes(const daq_conv_desc& d);
daq_status quantize_activation_check(const daq_conv_desc& d, const float* X);   // host only: can this X be quantized?
daq_status quantize_activation(const daq_conv_desc& d, const float* X, int8_t* qx_nhwc, int8_t* qx_cnhw, float* s_x,
                               void* ws, hipStream_t st, daq_schedule schedule);
daq_status quantize_filter(const daq_conv_desc& d, const float* W, int8_t* qw_packed, float* s_w, void* ws,
                           hipStream_t st);

// clip_search.hip
size_t clip_search_ws_bytes(const daq_conv_desc& d);

// conv_generic.hip: direct kernels, any descriptor
daq_status conv_fwd_generic(const daq_conv_desc& d, const int8_t* qx_nhwc, const int8_t* qw, const float* s_x,
                            const float* s_w, float* Y, int32_t* acc, hipStream_t st);
// With `bf16` the result pointer of a gradient routine (dX, dW) is bfloat16 storage: same product, rounded to nearest even.
daq_status conv_bwd_data_generic(const daq_conv_desc& d, const int8_t* qg, const float* s_g, const int8_t* qw,
                                 const float* s_w, float* dX, int32_t* acc, hipStream_t st, bool bf16 = false);
daq_status conv_bwd_filter_generic(const daq_conv_desc& d, const int8_t* qx, const float* s_x, const int8_t* vq,
                                   const float* s_chan, float* dW, int32_t* acc, hipStream_t st, bool bf16 = false);

// conv_mfma_*.hip: int8 MFMA kernels; *_supported() says whether a descriptor is covered
bool bwd_filter_mfma_supported(const daq_conv_desc& d);
size_t bwd_filter_mfma_ws_bytes(const daq_conv_desc& d);
daq_status conv_bwd_filter_mfma(const daq_conv_desc& d, const int8_t* qx, const float* s_x, const int8_t* vq,
                                const float* s_chan, float* dW, int32_t* acc, void* ws, hipStream_t st, bool bf16 = false);
bool bwd_data_mfma_supported(const daq_conv_desc& d);
daq_status conv_bwd_data_mfma(const daq_conv_desc& d, const int8_t* qg, const float* s_g, const int8_t* qw,
                              const float* s_w, float* dX, int32_t* acc, hipStream_t st, bool bf16 = false);
bool fwd_mfma_supported(const daq_conv_desc& d);
daq_status conv_fwd_mfma(const daq_conv_desc& d, const int8_t* qx_nhwc, const int8_t* qw, const float* s_x,
                         const float* s_w, float* Y, int32_t* acc, hipStream_t st);


// conv_mfma_dw32.hip: 3 x 3 unit-stride filter gradient on the 32x32x32 MFMA, operands staged through LDS
bool bwd_filter_lds_supported(const daq_conv_desc& d);
size_t bwd_filter_lds_ws_bytes(const daq_conv_desc& d);
// With `defer`, a K-split launch leaves its last stage (sum of the partial tiles, de-quantization) undone and
// describes it in *defer (blocks == 0: nothing is left) for a later kernel's extra workgroups, see dw_tail.h.
struct DwTail;
daq_status conv_bwd_filter_lds(const daq_conv_desc& d, const int8_t* qx, const float* s_x, const int8_t* vq,
                               const float* s_chan, float* dW, int32_t* acc, void* ws, hipStream_t st,
                               DwTail* defer = nullptr, bool bf16 = false);

// conv_mfma_halo.hip: halo-tile form of the channel-contracting kernel (unit stride; stride 2 for the data gradient)
bool bwd_data_halo_supported(const daq_conv_desc& d);
// With `tail` (blocks > 0), extra workgroups of the launch finish a deferred filter gradient.
// With `bf16`, dX points to bfloat16 storage (2 bytes per element) and receives the result rounded to nearest even.
daq_status conv_bwd_data_halo(const daq_conv_desc& d, const int8_t* qg, const float* s_g, const int8_t* qw,
                              const float* s_w, float* dX, int32_t* acc, hipStream_t st, const DwTail* tail = nullptr,
                              bool bf16 = false);
bool fwd_halo_supported(const daq_conv_desc& d);
daq_status conv_fwd_halo(const daq_conv_desc& d, const int8_t* qx_nhwc, const int8_t* qw, const float* s_x,
                         const float* s_w, float* Y, int32_t* acc, hipStream_t st);

// conv_depthwise.hip: groups == channels, both operands channel-major
bool depthwise_dx_supported(const daq_conv_desc& d);
daq_status conv_bwd_data_depthwise(const daq_conv_desc& d, const int8_t* qg, const float* s_g, const int8_t* qw,
                                   const float* s_w, float* dX, int32_t* acc, hipStream_t st, bool per_channel = false,
                                   bool bf16 = false);
bool depthwise_fwd_supported(const daq_conv_desc& d);
daq_status conv_fwd_depthwise(const daq_conv_desc& d, const int8_t* qx_cnhw, const int8_t* qw, const float* s_x,
                              const float* s_w, float* Y, int32_t* acc, hipStream_t st);
bool depthwise_dw_supported(const daq_conv_desc& d);
size_t depthwise_dw_ws_bytes(const daq_conv_desc& d);
daq_status conv_bwd_filter_depthwise(const daq_conv_desc& d, const int8_t* qx, const float* s_x, const int8_t* vq,
                                     const float* s_chan, float* dW, int32_t* acc, void* ws, hipStream_t st, bool bf16 = false);

}  // namespace daq
