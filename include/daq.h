/*
 * daq.h -- C ABI of the INT8 convolution backward path with Distribution
 * Adaptive gradient quantization (arXiv 2102.04782) for AMD MI355X (gfx950).
 *
 * One conv layer's backward pass (the paper's Algorithm 1) is three calls:
 *
 *     daq_quantize_grad        statistics, discriminator, clip values, the
 *                              vectorized (per-channel) and the global int8
 *                              copies of the output gradient dY
 *     daq_conv_bwd_filter_int8 q(G_W) = q(X') (x) vq(G'), vectorized de-quantization
 *     daq_conv_bwd_data_int8   q(G_X) = q(G) (.) q(W),    global de-quantization
 *
 * and the forward pass that saves q(X), q(W), s_X, s_W for them is
 *
 *     daq_conv_fwd_int8
 *
 * Conventions, valid for every entry point:
 *   - Every data pointer is DEVICE memory owned by the caller.  The library
 *     allocates nothing, never synchronises the stream and never copies a
 *     scalar to the host: scales are passed between calls as device pointers.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on it in order; the call returns before it completes.
 *   - `workspace` is caller-provided scratch of at least daq_workspace_bytes()
 *     bytes, 256-byte aligned, private to the call until the stream reaches
 *     its end.  Its previous contents do not matter.
 *   - The return value is the only error channel.  Arguments are validated on
 *     the host before anything is launched; on an error no output is touched.
 *   - fp32 tensors are dense NCHW / [Cout][Cin/groups][kH][kW].  int8 tensors
 *     use the layouts described by daq_layout_* below; bytes of those buffers
 *     that hold no element are written as zero by the producing call and must
 *     stay zero.
 *   - int8 buffers and the fp32 / int32 outputs of the data gradient and the forward pass must be
 *     16-byte aligned, every other fp32 tensor 4-byte aligned (the wider paths are taken when it is
 *     16-byte aligned); anything else is DAQ_ERR_INVALID_ARG.
 *   - Inputs are assumed finite (no NaN/Inf).
 */
#ifndef DAQ_H
#define DAQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Convolution problem, in the notation of the paper's method section:
 * X in (N, Cin, Hin, Win), W in (Cout, Cin/groups, kH, kW), Y and G = dY in (N, Cout, Hout, Wout). */
typedef struct {
    int32_t N, Cin, Hin, Win;
    int32_t Cout, kH, kW;
    int32_t strideH, strideW;
    int32_t padH, padW;
    int32_t dilH, dilW;
    int32_t groups;
} daq_conv_desc;

typedef enum {
    DAQ_OK = 0,
    DAQ_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, inconsistent descriptor, bad enum */
    DAQ_ERR_WORKSPACE = 2,   /* workspace missing, misaligned or smaller than daq_workspace_bytes() */
    DAQ_ERR_UNSUPPORTED = 3, /* valid problem the library has no kernel for (sizes beyond 2^31 elements) */
    DAQ_ERR_HIP = 4,         /* a HIP call or kernel launch reported an error */
    DAQ_ERR_SCRATCH_LIMIT = 5 /* daq_quantize_grad_noalloc: the problem needs more scratch than DAQ_STATIC_SCRATCH_BYTES */
} daq_status;

/* Rounding of the gradient quantizer (text after Eq. "suq": stochastic rounding for
 * gradients, nearest for weights and activations).  Nearest is ties-to-even. */
typedef enum { DAQ_ROUND_NEAREST = 0, DAQ_ROUND_STOCHASTIC = 1 } daq_round;

/* Channel classes of the gradient discriminator, Eq. "judge". */
enum { DAQ_CLASS_GAUSS = 0, DAQ_CLASS_INVT = 1 };

typedef enum {
    DAQ_OP_QUANTIZE_GRAD = 0, DAQ_OP_CONV_FWD = 1, DAQ_OP_CONV_BWD_DATA = 2, DAQ_OP_CONV_BWD_FILTER = 3,
    DAQ_OP_CONV_BWD = 4, /* both gradients in one call */
    DAQ_OP_CLIP_SEARCH = 5
} daq_op;

/* ---------------------------------------------------------------------------------------------
 * int8 tensor layouts
 *
 * Two families.  Which one a buffer uses, and its parameters, are a pure function of the
 * convolution descriptor; ask with daq_layout_*().
 *
 * DAQ_LAYOUT_NHWC -- channels innermost, the reduction axis of the data-gradient and forward
 *   products.  Element (n, c, h, w) is byte  ((n*H + h)*W + w) * c_pitch + c ;
 *   c_pitch = C rounded up to 16, bytes c >= C are zero.
 *
 * DAQ_LAYOUT_CNHW -- the paper's dimension transformation X -> X' in (Cin, N, H, W),
 *   G -> G' in (Cout, N, Hout, Wout): channel outermost, so the reduction axis (n, h, w) of the
 *   filter-gradient product is contiguous.  Images sit in slots of img_rows x row_pitch bytes that
 *   are at least as large as the image; the extra bytes are zero and provide the convolution's
 *   zero padding.  With  hh = h + org_h, ww = w + org_w  element (n, c, h, w) is byte
 *       c*chan_pitch + ((hh % phases_h)*phases_w + (ww % phases_w)) * plane_pitch + lead
 *         + (n*img_rows + hh / phases_h) * row_pitch + ww / phases_w .
 *   phases_* > 1 only for the saved activation of a strided convolution (one plane per stride
 *   phase, so every filter tap reads one plane at a constant offset).  The lead bytes in front of
 *   the first image of a plane and the bytes behind its last image are zero as well, and cover
 *   every position a filter tap can reach from a real element in either direction.
 * ------------------------------------------------------------------------------------------- */
typedef enum { DAQ_LAYOUT_NHWC = 0, DAQ_LAYOUT_CNHW = 1 } daq_layout_kind;

typedef struct {
    int32_t kind;       /* daq_layout_kind */
    int32_t C, N, H, W; /* logical extents of the tensor */
    int64_t bytes;      /* size of the buffer */
    int32_t c_pitch;    /* NHWC only */
    int32_t img_rows, row_pitch; /* CNHW only, as are the fields below */
    int32_t phases_h, phases_w;
    int32_t org_h, org_w;
    int64_t chan_pitch, plane_pitch, lead;
} daq_layout;

/* Layout of the per-channel quantized gradient vq(G') (always CNHW). */
daq_status daq_layout_vq(const daq_conv_desc* desc, daq_layout* out);
/* Layout of the globally quantized gradient q(G): NHWC, or CNHW for depthwise layers (groups == Cin == Cout). */
daq_status daq_layout_qg(const daq_conv_desc* desc, daq_layout* out);
/* Layout of the saved activation q(X) consumed by the forward and data-gradient side (NHWC). */
daq_status daq_layout_qx_nhwc(const daq_conv_desc* desc, daq_layout* out);
/* Layout of the saved, dimension-transformed activation q(X') consumed by the filter gradient (CNHW). */
daq_status daq_layout_qx_cnhw(const daq_conv_desc* desc, daq_layout* out);

/* Packed int8 filter q(W): three copies in one buffer.
 *   plain  at off_plain: [Cout][Cin/groups][kH][kW]
 *   fwd    at off_fwd  : [kH*kW][Cout][cig_pitch]   (input channel of the group innermost)
 *   bwd    at off_bwd  : [kH*kW][Cin][cog_pitch]    (output channel of the group innermost)
 * cig_pitch / cog_pitch = Cin/groups, Cout/groups rounded up to 16; padding bytes are zero.
 * For groups == 1 two more copies hold the filter in the register order of the matrix-core kernels
 * ("fragment order"), so that a wavefront fetches a 32-row x 32-byte operand tile as one contiguous KiB:
 *   fwd_frag at off_fwd_frag: rows = output channels, k = input channels
 *   bwd_frag at off_bwd_frag: rows = input channels,  k = output channels
 * element (tap, row, k) of a copy with RB = ceil(rows/32) row blocks and T = kH*kW taps is byte
 *   ((((k/64)*T + tap)*RB + row/32)*2 + (k%64)/32)*1024 + (((k%32)/16)*32 + row%32)*16 + k%16 ;
 * rows and k are padded with zeros to multiples of 32 and 64.  Both offsets equal `bytes` when groups > 1. */
typedef struct {
    int64_t bytes;
    int64_t off_plain, off_fwd, off_bwd;
    int32_t cig_pitch, cog_pitch;
    int64_t off_fwd_frag, off_bwd_frag;
} daq_wpack_layout;
daq_status daq_layout_qw(const daq_conv_desc* desc, daq_wpack_layout* out);

/* Output spatial size of the convolution; 0 if the descriptor is invalid. */
int32_t daq_out_h(const daq_conv_desc* desc);
int32_t daq_out_w(const daq_conv_desc* desc);

/* Scratch bytes an entry point needs for this problem (host function, no GPU call).
 * Returns 0 for an invalid descriptor or op. */
size_t daq_workspace_bytes(daq_op op, const daq_conv_desc* desc);

/* ---------------------------------------------------------------------------------------------
 * daq_quantize_grad -- Algorithm 1, the per-channel loop and the two quantizations.
 *
 * For every output channel c of dY (fp32 [N][Cout][Hout][Wout]):
 *   |g|max_c, sigma_c (population std about the channel mean, fp64 accumulation),
 *   P_c = #{|g| > sigma_c} / (N*Hout*Wout),
 *   class_c = GAUSS if P_c > lambda else INVT                         (Eq. "judge"),
 *   s_c = |g|max_c                                   for GAUSS        (Eq. "gaus"),
 *   s_c = (1 - k*A) * s_state[c] + A * |g|max_c      for INVT         (Eq. "fats"),
 *         where a non-positive s_state[c] ("no history") or result is replaced by |g|max_c,
 *   s_state[c] <- s_c (both classes).
 * Then  vq = Q(dY, s_c) per channel,  qg = Q(dY, s_global),  s_global = max_c |g|max_c,
 * Q being Eq. "suq" evaluated in fp32 as round(clamp(x * (127/s), -127, 127)).
 * A scale below 2^-100 is reported as 0 and produces all-zero codes.
 * Stochastic rounding: with fmix32 the 32-bit finalizer of MurmurHash3 and
 *   key = fmix32(seed_lo ^ fmix32(seed_hi ^ 0x9E3779B9)),
 * element i (its NCHW index) hashes once, h = fmix32(i ^ key); vq draws u = (h >> 16) * 2^-16, qg draws
 * u = (h & 0xFFFF) * 2^-16, and a copy rounds up iff frac(x*127/s) > u.
 *
 *   dY        in   fp32 NCHW
 *   s_state   i/o  fp32 [Cout]  clip values of the previous iteration, replaced by this iteration's
 *   vq        out  int8, layout daq_layout_vq
 *   qg        out  int8, layout daq_layout_qg
 *   s_chan    out  fp32 [Cout];  s_global out fp32 [1];  cls out u8 [Cout]
 *   stats     out  optional (may be NULL) fp32 [Cout][4] = |g|max, mean, sigma, P
 * Hyper-parameters of the paper: k = 1, A = 0.8, lambda = 0.3.
 *
 * Schedule (results do not depend on it, see daq_schedule): three sweeps over dY - statistics;
 * count + qg; vq.  For gradients of 8 Mi elements and more the second sweep also writes vq under a
 * class guessed from |g|max / sigma, and the third only redoes the channels whose guess was wrong.
 * ------------------------------------------------------------------------------------------- */
daq_status daq_quantize_grad(const daq_conv_desc* desc, const float* dY, float* s_state, float k, float A,
                             float lambda, daq_round mode, uint64_t seed, int8_t* vq, int8_t* qg, float* s_chan,
                             float* s_global, uint8_t* cls, float* stats, void* workspace, size_t workspace_bytes,
                             void* stream);

/* ---------------------------------------------------------------------------------------------
 * daq_quantize_grad_scheme -- daq_quantize_grad with the rule for the per-channel clip values s_c
 * chosen by the caller: Algorithm 1, or one of the three variants the experiments section compares
 * it with ("Ablation study").  qg and s_global are the same under every scheme.
 *   DAQ_SCHEME_DAQ  Algorithm 1 (what daq_quantize_grad computes).
 *   DAQ_SCHEME_GQ   the baseline, global quantization: s_c = max over channels of |g|max_c, so the
 *                   copy for dW is quantized like the copy for dX.
 *   DAQ_SCHEME_GVQ  vectorized quantization with the baseline's rule per channel: s_c = |g|max_c.
 *   DAQ_SCHEME_MCS  Magnitude-aware Clipping on the layer-wise gradient: |g|max, sigma and the tail
 *                   mass P = #{|g| > sigma} / (N*Cout*Hout*Wout) of the whole tensor taken as one
 *                   population give one class (Eq. "judge") and one clip value (Eq. "gaus" / Eq.
 *                   "fats") that every channel uses.  The history is s_state[0].
 * s_state[c] <- s_c under every scheme.  cls and stats: under GQ and GVQ the per-channel values of
 * Algorithm 1 (they decide nothing there); under MCS every channel's entry holds the layer's.
 * All other arguments, the workspace and the error codes as for daq_quantize_grad; an unknown scheme
 * is DAQ_ERR_INVALID_ARG.
 * ------------------------------------------------------------------------------------------- */
typedef enum { DAQ_SCHEME_DAQ = 0, DAQ_SCHEME_GQ = 1, DAQ_SCHEME_GVQ = 2, DAQ_SCHEME_MCS = 3 } daq_scheme;
daq_status daq_quantize_grad_scheme(const daq_conv_desc* desc, const float* dY, float* s_state, float k, float A,
                                    float lambda, daq_round mode, uint64_t seed, daq_scheme scheme, int8_t* vq,
                                    int8_t* qg, float* s_chan, float* s_global, uint8_t* cls, float* stats,
                                    void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * daq_quantize_grad_ex -- the quantizer with every option explicit; the three entry points around it
 * forward to it.  The library reads no environment variable and keeps no tuning state: which kernels
 * run is a function of the arguments alone.
 *
 *   opts->scheme    daq_scheme (rule for the per-channel clip values)
 *   opts->schedule  daq_schedule: how the sweeps over dY are shared out among the launches.  The
 *                   results are the same bits under every schedule.
 *                     DAQ_SCHEDULE_AUTO          the library picks by size (what the other entry points do)
 *                     DAQ_SCHEDULE_THREE_SWEEPS  statistics; count + qg; vq
 *                     DAQ_SCHEDULE_EARLY_COPY    the counting sweep also writes vq under a guessed class
 *                     DAQ_SCHEDULE_CHANNEL_RESIDENT  one workgroup per channel keeps the channel in registers,
 *                                                so that statistics, count, decision and vq take ONE read of dY;
 *                                                a second launch writes qg.  For channels of at most 65536
 *                                                elements (N*Hout*Wout; 16384 where Hout*Wout is not a multiple
 *                                                of four or dY is not a 16-byte aligned fp32 tensor) whose int8
 *                                                plane is at most 96 KiB, under Algorithm 1's rule with an NHWC
 *                                                global copy; taken by default where it applies.
 *                   A schedule the layer cannot take (the early copy needs Algorithm 1's rule, an NHWC
 *                   global copy and an unsplit channel-major layout with rows of even length) falls
 *                   back to three sweeps.
 *   opts->dy_bf16   0: dY is fp32; 1: dY is bfloat16 (see daq_quantize_grad_bf16)
 *   opts->reserved  must be 0
 *   opts == NULL    Algorithm 1, automatic schedule, fp32
 * Other arguments, the workspace and the error codes as for daq_quantize_grad; an unknown scheme or
 * schedule is DAQ_ERR_INVALID_ARG.
 * ------------------------------------------------------------------------------------------- */
typedef enum {
    DAQ_SCHEDULE_AUTO = 0, DAQ_SCHEDULE_THREE_SWEEPS = 1, DAQ_SCHEDULE_EARLY_COPY = 2, DAQ_SCHEDULE_CHANNEL_RESIDENT = 3
} daq_schedule;
typedef struct {
    int32_t scheme, schedule, dy_bf16, reserved;
} daq_quantize_opts;
daq_status daq_quantize_grad_ex(const daq_conv_desc* desc, const void* dY, float* s_state, float k, float A, float lambda,
                                daq_round mode, uint64_t seed, const daq_quantize_opts* opts, int8_t* vq, int8_t* qg,
                                float* s_chan, float* s_global, uint8_t* cls, float* stats, void* workspace,
                                size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * daq_quantize_grad_split -- daq_quantize_grad_ex on two streams (Algorithm 1's two int8 copies have
 * different consumers: Eq. "gx" reads qg, Eq. "gw" reads vq).  In a backward pass only the data
 * gradient is on the critical path: the next layer's gradient waits for it, nothing waits for the
 * filter gradient.  This entry point keeps on `stream` exactly the launches qg and s_global need,
 * and moves the others to `side_stream`, which first waits (hipStreamWaitEvent on an event the
 * library records on `stream`; one event per device, created at the first call and kept) for the
 * launches before them.  When the call returns
 *   qg, s_global                            are complete in the order of `stream`,
 *   vq, s_chan, cls, stats, s_state         are complete in the order of `side_stream`:
 * launch the data gradient on `stream` and the filter gradient on `side_stream`, with no further
 * synchronisation between the two.  The caller orders the next use of s_state, of the outputs and
 * of the workspace (the next call for this layer) behind BOTH streams.  Results: the same bits as
 * daq_quantize_grad_ex.  side_stream NULL or equal to stream: daq_quantize_grad_ex.  Both streams
 * belong to the current device.  A layer whose global copy is channel-major (depthwise) keeps every
 * launch on `stream`, and `side_stream` waits for those that the per-channel outputs need.  Other arguments, workspace and
 * error codes as for daq_quantize_grad_ex; a failing event call is DAQ_ERR_HIP.
 * ------------------------------------------------------------------------------------------- */
daq_status daq_quantize_grad_split(const daq_conv_desc* desc, const void* dY, float* s_state, float k, float A, float lambda,
                                   daq_round mode, uint64_t seed, const daq_quantize_opts* opts, int8_t* vq, int8_t* qg,
                                   float* s_chan, float* s_global, uint8_t* cls, float* stats, void* workspace,
                                   size_t workspace_bytes, void* stream, void* side_stream);

/* ---------------------------------------------------------------------------------------------
 * daq_quantize_grad_from_stats -- Algorithm 1 from its second step on, for a producer of dY that
 * already has the channel statistics ("Infer |g|max and sigma" is then no sweep of its own; the
 * paper notes that the two quantizations "can be easily optimized with kernel fusion").  A kernel
 * that writes dY (the backward of a normalisation or activation layer) can reduce, per channel c over
 * all of (n, h, w),
 *   ch_absmax[c] = max |g|          fp32, device, [Cout]
 *   ch_sum[c]    = sum g            fp64, device, [Cout], 8-byte aligned
 *   ch_sumsq[c]  = sum g*g          fp64, device, [Cout], 8-byte aligned   (g widened to fp64 first)
 * on its way; the three arrays are read, never written.  From them mu = sum/M, sigma =
 * fp32(sqrt(max(0, sumsq/M - mu*mu))) in fp64, exactly as the other entry points derive them from
 * their own sums, and everything after (tail mass, Eq. "judge", Eq. "gaus"/"fats", both int8 copies)
 * is the same code.  One sweep over dY remains: it counts and writes both copies (the per-channel
 * one under a guessed class, redone for the channels whose guess was wrong), 6 bytes per element
 * instead of 10; layers whose copies that sweep cannot write (channel-major global copy, ablation
 * rules, rows the vector path does not serve) and opts->schedule = DAQ_SCHEDULE_THREE_SWEEPS keep a
 * counting and a packing sweep.  Results: those of daq_quantize_grad_ex bit for bit when the
 * statistics are the channel's (fp64 sums taken in another order can differ in their last bits;
 * sigma is rounded to fp32, so that shows only where an element's magnitude or a channel's count
 * sits exactly on the threshold); for other values, the algorithm's result for those statistics.
 * stream / side_stream as for daq_quantize_grad_split (side_stream may be NULL).  Null or
 * misaligned statistics: DAQ_ERR_INVALID_ARG; other arguments, workspace and error codes as for
 * daq_quantize_grad_ex.
 * ------------------------------------------------------------------------------------------- */
daq_status daq_quantize_grad_from_stats(const daq_conv_desc* desc, const void* dY, const float* ch_absmax,
                                        const double* ch_sum, const double* ch_sumsq, float* s_state, float k, float A,
                                        float lambda, daq_round mode, uint64_t seed, const daq_quantize_opts* opts,
                                        int8_t* vq, int8_t* qg, float* s_chan, float* s_global, uint8_t* cls, float* stats,
                                        void* workspace, size_t workspace_bytes, void* stream, void* side_stream);

/* ---------------------------------------------------------------------------------------------
 * daq_quantize_grad_noalloc -- daq_quantize_grad for callers that cannot allocate device memory and
 * so cannot provide a workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  The scratch of the three sweeps (statistics and count partials) lives in a
 * fixed array of DAQ_STATIC_SCRATCH_BYTES in the library's device image instead; the call allocates
 * and frees nothing.  Same kernels, same results, bit for bit, as daq_quantize_grad.
 *
 *   - A problem whose daq_workspace_bytes(DAQ_OP_QUANTIZE_GRAD) exceeds DAQ_STATIC_SCRATCH_BYTES is
 *     refused with DAQ_ERR_SCRATCH_LIMIT before anything is launched (every layer of ResNet-50 at
 *     batch 64 and MobileNetV2 at batch 128 needs less than 0.4 MiB).
 *   - Each GPU has its own copy of the array; the one of the CURRENT device is used, so the device
 *     that `stream` belongs to must be current.  Its address is looked up on the first call on a
 *     device (not an allocation; make that first call outside graph capture).
 *   - All calls on one GPU share the array: two calls whose kernels overlap in time - different
 *     streams, or threads - race.  Calls on one stream are ordered and safe.  Nothing in the array
 *     needs clearing between calls.
 *   arguments as for daq_quantize_grad, without the workspace
 * ------------------------------------------------------------------------------------------- */
#define DAQ_STATIC_SCRATCH_BYTES (1 << 20)
daq_status daq_quantize_grad_noalloc(const daq_conv_desc* desc, const float* dY, float* s_state, float k, float A,
                                     float lambda, daq_round mode, uint64_t seed, int8_t* vq, int8_t* qg, float* s_chan,
                                     float* s_global, uint8_t* cls, float* stats, void* stream);

/* ---------------------------------------------------------------------------------------------
 * daq_quantize_grad_bf16 -- daq_quantize_grad_scheme for an output gradient stored as bfloat16
 * (what a mixed-precision backward pass hands over).  A bfloat16 value is the upper half of an fp32
 * pattern, so widening is exact: every output equals, bit for bit, what daq_quantize_grad_scheme
 * returns for the widened tensor - statistics, classes, clip values, both int8 copies, and the
 * random numbers of stochastic rounding (still indexed by the NCHW position).  The three sweeps
 * read 2 instead of 4 bytes per element.
 *
 *   dY_bf16   in   bfloat16 NCHW, 2-byte aligned (8-byte alignment lets the packing pass load
 *                  whole vectors)
 *   all other arguments, the workspace and the error codes as for daq_quantize_grad_scheme
 * ------------------------------------------------------------------------------------------- */
daq_status daq_quantize_grad_bf16(const daq_conv_desc* desc, const uint16_t* dY_bf16, float* s_state, float k, float A,
                                  float lambda, daq_round mode, uint64_t seed, daq_scheme scheme, int8_t* vq,
                                  int8_t* qg, float* s_chan, float* s_global, uint8_t* cls, float* stats,
                                  void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * daq_conv_fwd_int8 -- forward pass of the quantized layer (dataflow figure; the inputs that
 * Algorithm 1 requires).  s_x = max|X|, s_w = max|W| (global quantization, nearest rounding),
 * Y = (int32 conv of the codes) * (s_x/127) * (s_w/127).
 *
 *   X, W        in   fp32
 *   qx_nhwc     out  int8 daq_layout_qx_nhwc      qx_cnhw out int8 daq_layout_qx_cnhw
 *   qw_packed   out  int8 daq_layout_qw
 *   s_x, s_w    out  fp32 [1] each
 *   Y           out  fp32 NCHW
 *   acc_out     out  optional (may be NULL) int32 NCHW raw accumulators, for verification
 * ------------------------------------------------------------------------------------------- */
daq_status daq_conv_fwd_int8(const daq_conv_desc* desc, const float* X, const float* W, int8_t* qx_nhwc,
                             int8_t* qx_cnhw, int8_t* qw_packed, float* s_x, float* s_w, float* Y, int32_t* acc_out,
                             void* workspace, size_t workspace_bytes, void* stream);

/* daq_conv_fwd_int8 with the schedule of its activation quantizer explicit: DAQ_SCHEDULE_EARLY_COPY
 * writes both layouts of q(X) in one sweep over X (taken by default from 8 Mi elements on, where
 * the channel-major layout is unsplit), DAQ_SCHEDULE_THREE_SWEEPS (and DAQ_SCHEDULE_CHANNEL_RESIDENT, which has no
 * forward form) one sweep per layout.  Same bits. */
daq_status daq_conv_fwd_int8_ex(const daq_conv_desc* desc, const float* X, const float* W, int8_t* qx_nhwc,
                                int8_t* qx_cnhw, int8_t* qw_packed, float* s_x, float* s_w, float* Y, int32_t* acc_out,
                                daq_schedule schedule, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * daq_conv_bwd_data_int8 -- Eq. "gx" on int8 codes with int32 accumulation:
 *   acc[n,ci,h,w] = sum over (co in the group, kh, kw) of qg[n,co,ho,wo] * qW[co,ci,kh,kw]
 *   with ho*strideH + kh*dilH - padH == h (same for w), ho, wo inside the output;
 *   dX = acc * ((s_w/127) * (s_global/127)).
 * Accumulators wrap modulo 2^32 (not reachable below 133144 taps per output).
 *
 *   qg        in   int8 daq_layout_qg        s_global in fp32 [1]
 *   qw_packed in   int8 daq_layout_qw        s_w      in fp32 [1]
 *   dX        out  fp32 NCHW
 *   acc_out   out  optional int32 NCHW
 * ------------------------------------------------------------------------------------------- */
daq_status daq_conv_bwd_data_int8(const daq_conv_desc* desc, const int8_t* qg, const float* s_global,
                                  const int8_t* qw_packed, const float* s_w, float* dX, int32_t* acc_out,
                                  void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * daq_conv_bwd_filter_int8 -- Eq. "gw" on int8 codes with the vectorized de-quantization:
 *   acc[co,cl,kh,kw] = sum over (n,ho,wo) of qX[n,ci,ho*strideH+kh*dilH-padH, wo*strideW+kw*dilW-padW] * vq[n,co,ho,wo]
 *   dW[co,...] = acc[co,...] * ((s_x/127) * (s_chan[co]/127)).
 *
 *   qx_cnhw   in   int8 daq_layout_qx_cnhw   s_x    in fp32 [1]
 *   vq        in   int8 daq_layout_vq        s_chan in fp32 [Cout]
 *   dW        out  fp32 [Cout][Cin/groups][kH][kW]
 *   acc_out   out  optional int32, same shape
 * ------------------------------------------------------------------------------------------- */
daq_status daq_conv_bwd_filter_int8(const daq_conv_desc* desc, const int8_t* qx_cnhw, const float* s_x,
                                    const int8_t* vq, const float* s_chan, float* dW, int32_t* acc_out,
                                    void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * daq_conv_bwd_int8 -- the last two steps of Algorithm 1 (Eq. "gw" with the vectorized
 * de-quantization and Eq. "gx" with the global one) in one call: the same arguments, the same
 * arithmetic and the same results, bit for bit, as daq_conv_bwd_filter_int8 followed by
 * daq_conv_bwd_data_int8.  The two gradients do not depend on each other, which the library uses to
 * save a launch: where the filter gradient splits its contraction axis across workgroups, the sum
 * of the partial tiles and the de-quantization are done by extra workgroups of the data-gradient
 * kernel instead of a launch of their own.
 *
 *   arguments as in the two calls above; dW_acc / dX_acc are their optional acc_out
 *   workspace: daq_workspace_bytes(DAQ_OP_CONV_BWD, desc)
 * ------------------------------------------------------------------------------------------- */
daq_status daq_conv_bwd_int8(const daq_conv_desc* desc, const int8_t* qx_cnhw, const float* s_x, const int8_t* vq,
                             const float* s_chan, float* dW, int32_t* dW_acc, const int8_t* qg, const float* s_global,
                             const int8_t* qw_packed, const float* s_w, float* dX, int32_t* dX_acc, void* workspace,
                             size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * daq_conv_bwd_data_int8_bf16 / daq_conv_bwd_filter_int8_bf16 -- the two gradients with a narrow
 * result: the same int32 accumulators and the same fp32 products acc * ((s_w/127) * (s_global/127))
 * and acc * ((s_x/127) * (s_chan[co]/127)), stored as bfloat16 (round to nearest, ties to even).
 * An option beside the method, not part of it: Algorithm 1 returns full-precision gradients; the
 * data gradient's fp32 result is the largest stream of the backward pass (4 bytes per input
 * element), and a consumer that takes bf16 halves it.  Every layer daq_conv_bwd_data_int8 /
 * daq_conv_bwd_filter_int8 serve is served, by the same kernels.
 *
 *   dX_bf16   out  bfloat16 NCHW, 16-byte aligned
 *   dW_bf16   out  bfloat16 [Cout][Cin/groups][kH][kW], 2-byte aligned
 *   other arguments and the workspace as for the fp32 entry points
 * ------------------------------------------------------------------------------------------- */
daq_status daq_conv_bwd_data_int8_bf16(const daq_conv_desc* desc, const int8_t* qg, const float* s_global,
                                       const int8_t* qw_packed, const float* s_w, uint16_t* dX_bf16, void* workspace,
                                       size_t workspace_bytes, void* stream);
daq_status daq_conv_bwd_filter_int8_bf16(const daq_conv_desc* desc, const int8_t* qx_cnhw, const float* s_x,
                                         const int8_t* vq, const float* s_chan, uint16_t* dW_bf16, void* workspace,
                                         size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * daq_conv_bwd_data_int8_chan -- data gradient of a depthwise layer (groups = Cin = Cout, the
 * MobileNetV2 paragraph's layers) from the PER-CHANNEL copy of dY.  There channel c of the data
 * gradient is a function of channel c of dY alone, so the vectorized quantization and its
 * de-quantization carry over from Eq. "gw" to Eq. "gx":
 *   acc as in daq_conv_bwd_data_int8 with vq in the place of qg;
 *   dX[n,c,:,:] = acc[n,c,:,:] * ((s_w/127) * (s_chan[c]/127)).
 * An option beside Algorithm 1, which takes the global |g|max for the data gradient: channels of
 * small spread keep their resolution, and a caller that uses it needs no global copy for the layer.
 * DAQ_ERR_UNSUPPORTED for any other layer, and for depthwise layers the channel-major kernels do
 * not serve (filters above 7 x 7, strides that are not one power of two for both axes).
 *
 *   vq        in   int8 daq_layout_vq        s_chan in fp32 [Cout]
 *   other arguments, alignment and the workspace as for daq_conv_bwd_data_int8
 * ------------------------------------------------------------------------------------------- */
daq_status daq_conv_bwd_data_int8_chan(const daq_conv_desc* desc, const int8_t* vq, const float* s_chan,
                                       const int8_t* qw_packed, const float* s_w, float* dX, int32_t* acc_out,
                                       void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * 3-D convolution layers (the video-classification experiment: "treating depth dimension in the same
 * way as height and width").  X in (N, Cin, Din, Hin, Win), W in (Cout, Cin/groups, kD, kH, kW), Y and
 * G = dY in (N, Cout, Do, Ho, Wo); fp32 tensors are dense in that order.  Algorithm 1 is unchanged:
 * its statistics run over all of (n, d, h, w), so the quantizer is the 2-D one on the gradient viewed
 * as (N, Cout, Do*Ho, Wo), and the two gradients are Eq. "gx" / Eq. "gw" with one more spatial axis.
 *
 * int8 layouts: those of two 2-D "carrier" problems, daq_conv3d_carriers():
 *   cx  describes the activation side: daq_layout_qx_nhwc(cx) / daq_layout_qx_cnhw(cx) are the layouts of q(X);
 *   cg  describes the gradient side:   daq_layout_vq(cg) / daq_layout_qg(cg) are the layouts of vq and qg.
 * Return value 1: the layer IS the 2-D problem cx == cg on reinterpreted tensors - a filter with kH = kW = 1 at unit
 * stride and no padding in height and width (time-only filters, pointwise layers: depth becomes the row axis, a whole
 * frame the column axis), or a volume of depth one - and every 3-D entry point forwards to its 2-D counterpart, the
 * matrix-core kernels included; q(W) is then packed as daq_layout_qw(cx).  Return value 0: any other layer; the
 * carriers are 1 x 1 problems that see (N, Cin, Din*Hin, Win) and (N, Cout, Do*Ho, Wo), and the products run on
 * direct integer kernels (4-wide int8 dot products where the shapes allow; exact; far from the matrix-core rate).
 * q(W) then holds the codes three times, each part rounded up to 256 bytes and zero where it holds no code: the
 * plain [Cout][Cin/groups][kD][kH][kW] array, [tap][Cout][Cin/groups rounded up to 16] and
 * [tap][Cin][Cout/groups rounded up to 16], tap = (kd*kH + kh)*kW + kw.  -1: invalid descriptor or sizes beyond
 * 2^31 elements.
 *
 * Entry points: arguments, alignment, error codes and results as for the 2-D entry point of the same name, with
 * workspaces of daq_conv3d_workspace_bytes(op, desc) and q(W) buffers of daq_conv3d_qw_bytes(desc).
 * ------------------------------------------------------------------------------------------- */
typedef struct {
    int32_t N, Cin, Din, Hin, Win;
    int32_t Cout, kD, kH, kW;
    int32_t strideD, strideH, strideW;
    int32_t padD, padH, padW;
    int32_t dilD, dilH, dilW;
    int32_t groups;
} daq_conv3d_desc;
int32_t daq_conv3d_out_d(const daq_conv3d_desc* desc);
int32_t daq_conv3d_out_h(const daq_conv3d_desc* desc);
int32_t daq_conv3d_out_w(const daq_conv3d_desc* desc);
int32_t daq_conv3d_carriers(const daq_conv3d_desc* desc, daq_conv_desc* cx, daq_conv_desc* cg);
int64_t daq_conv3d_qw_bytes(const daq_conv3d_desc* desc);
size_t daq_conv3d_workspace_bytes(daq_op op, const daq_conv3d_desc* desc);
daq_status daq_quantize_grad3d(const daq_conv3d_desc* desc, const void* dY, float* s_state, float k, float A, float lambda,
                               daq_round mode, uint64_t seed, const daq_quantize_opts* opts, int8_t* vq, int8_t* qg,
                               float* s_chan, float* s_global, uint8_t* cls, float* stats, void* workspace,
                               size_t workspace_bytes, void* stream);
daq_status daq_conv3d_fwd_int8(const daq_conv3d_desc* desc, const float* X, const float* W, int8_t* qx_nhwc, int8_t* qx_cnhw,
                               int8_t* qw, float* s_x, float* s_w, float* Y, int32_t* acc_out, void* workspace,
                               size_t workspace_bytes, void* stream);
daq_status daq_conv3d_bwd_data_int8(const daq_conv3d_desc* desc, const int8_t* qg, const float* s_global, const int8_t* qw,
                                    const float* s_w, float* dX, int32_t* acc_out, void* workspace, size_t workspace_bytes,
                                    void* stream);
daq_status daq_conv3d_bwd_filter_int8(const daq_conv3d_desc* desc, const int8_t* qx_cnhw, const float* s_x, const int8_t* vq,
                                      const float* s_chan, float* dW, int32_t* acc_out, void* workspace,
                                      size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * daq_clip_search -- the objective behind the Magnitude-aware Clipping Strategy, minimised by search.
 * For every output channel c of dY and every candidate clip value
 *     s_j = |g|max_c * (j / J),   j = 1 .. J   (fp32; s_J = |g|max_c),
 * the magnitude-weighted quantization error of Eq. "e" for the given alpha,
 *     E_c(s_j) = (1/M) * sum over (n, h, w) of  |g - g^| * exp(alpha * |g|),    M = N*Hout*Wout,
 *     g^ = round(clamp(g * (127/s_j), -127, 127)) * (s_j/127)      (Eq. "suq", nearest rounding, fp32),
 * with the difference, the weight and the sum in fp64; then best_j[c] = the j of the smallest error (the smallest j
 * among equals) and best_s[c] = s_{best_j}.  A channel whose |g|max is below 2^-100 has all errors equal and best_j = 1.
 * Not a step of Algorithm 1, whose clip values come from the closed-form rules that this objective led to (alpha does
 * not appear there): an analysis tool for comparing the two on real gradients.
 *
 *   dY      in   fp32 NCHW (Cout channels), 4-byte aligned
 *   alpha   in   >= 0 (alpha * |g|max above about 700 overflows the fp64 weights);   J in 1 .. 64
 *   err     out  optional (may be NULL) fp64 [Cout][J], 8-byte aligned
 *   best_s  out  fp32 [Cout];   best_j out int32 [Cout]
 *   workspace: daq_workspace_bytes(DAQ_OP_CLIP_SEARCH, desc)
 * fp64 sums are taken in a fixed order (same bits in every run) that differs from a sequential sum: errors agree with
 * a sequential evaluation to about 1e-12 relative.
 * ------------------------------------------------------------------------------------------- */
daq_status daq_clip_search(const daq_conv_desc* desc, const float* dY, float alpha, int32_t J, double* err, float* best_s,
                           int32_t* best_j, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Measurement aid (not part of the method).  Between daq_prof_begin() and daq_prof_end() every
 * kernel the library launches is bracketed by a HIP event pair on its stream.  daq_prof_end()
 * waits for those events and fills one row per distinct kernel name.  The list of pending event
 * pairs is the only state the library keeps between calls; it is guarded by a mutex, and while no
 * measurement is open the entry points do not touch it.
 * ------------------------------------------------------------------------------------------- */
typedef struct {
    char name[64];
    double total_ms;
    int32_t launches;
} daq_prof_row;
daq_status daq_prof_begin(void);
daq_status daq_prof_end(daq_prof_row* rows, int32_t max_rows, int32_t* n_rows);

/* Machine ceilings, for pricing the kernels against what this GPU delivers rather than against data-sheet peaks only.
 * Both enqueue one kernel on `stream` and return at once; the caller times them (events around the call).
 *   daq_ceiling_mfma_i8: `blocks` workgroups of four waves, each wave `iters` x 4 independent 32x32x32 int8 matrix-core
 *     multiply-accumulates on register operands; *ops receives the int8 operations (2 per multiply-add) of the launch.
 *   daq_ceiling_stream: mode 0 reads `bytes` of src, mode 1 writes `bytes` to dst, mode 2 copies src to dst, as 16-byte
 *     accesses from `blocks` workgroups.  src / dst are device memory, 16-byte aligned.
 *   sink: 4 bytes of device memory the kernels may write (never in practice; it keeps their work alive). */
daq_status daq_ceiling_mfma_i8(int32_t blocks, int32_t iters, void* sink, double* ops, void* stream);
daq_status daq_ceiling_stream(int32_t mode, const void* src, void* dst, size_t bytes, int32_t blocks, void* sink,
                              void* stream);

/* Human-readable name of a status code (static storage). */
const char* daq_status_string(daq_status s);

#ifdef __cplusplus
}
#endif
#endif /* DAQ_H */
