/*
 * daq_ref.c -- CPU oracle for the INT8 convolution backward pass of
 * "Distribution Adaptive INT8 Quantization for Training CNNs" (arXiv 2102.04782).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct
 * statement of what the hot path computes, written from the paper.  Only the
 * test-suite, the smoke check and the benchmark's cpu_baseline leg may call it.
 * It shares no code, header, table or helper with the HIP library.
 *
 * Every tensor is host memory.  int8 tensors are indexed logically (NCHW for
 * activations/gradients, [Cout][Cin/groups][kH][kW] for filters) whatever the
 * device library chooses for its own buffers.
 *
 * Arithmetic conventions (the readings taken where the paper is silent are
 * listed next to each function):
 *   - statistics are accumulated in fp64 and rounded once to fp32;
 *   - every decision that yields an integer (a code, a count, a class) is taken
 *     in fp32 with the operation order written here, no fused multiply-add
 *     (build with -ffp-contract=off);
 *   - integer accumulators are summed in int64, then wrapped to int32
 *     (two's complement) and an overflow flag is raised if wrapping changed them.
 *
 * OpenMP is used on outermost independent loops only (channels, output rows);
 * no blocking, fusion or reordering beyond the definitions.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define REF_OK 0
#define REF_BAD_ARG 1

#define REF_GAUSS 0 /* bell-shaped channel          (discriminator, Eq. "judge") */
#define REF_INVT 1  /* sharp / long-tailed channel  (Inverted-T)                 */

#define REF_ROUND_NEAREST 0
#define REF_ROUND_STOCHASTIC 1

/* A scale below this is treated as "the tensor is all zero": codes 0, scale 0. */
#define REF_TINY_SCALE 7.888609052210118e-31f /* 2^-100 */

typedef struct {
    int N, Cin, Hin, Win;
    int Cout, kH, kW;
    int strideH, strideW;
    int padH, padW;
    int dilH, dilW;
    int groups;
} ref_conv_desc;

int daq_ref_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int out_dim(int in, int pad, int dil, int k, int stride) {
    int eff = dil * (k - 1) + 1;
    int span = in + 2 * pad - eff;
    if (span < 0) return 0;
    return span / stride + 1;
}

int daq_ref_out_h(const ref_conv_desc* d) { return out_dim(d->Hin, d->padH, d->dilH, d->kH, d->strideH); }
int daq_ref_out_w(const ref_conv_desc* d) { return out_dim(d->Win, d->padW, d->dilW, d->kW, d->strideW); }

static int desc_ok(const ref_conv_desc* d) {
    if (!d) return 0;
    if (d->N <= 0 || d->Cin <= 0 || d->Hin <= 0 || d->Win <= 0 || d->Cout <= 0) return 0;
    if (d->kH <= 0 || d->kW <= 0 || d->strideH <= 0 || d->strideW <= 0) return 0;
    if (d->padH < 0 || d->padW < 0 || d->dilH <= 0 || d->dilW <= 0 || d->groups <= 0) return 0;
    if (d->Cin % d->groups || d->Cout % d->groups) return 0;
    if (daq_ref_out_h(d) <= 0 || daq_ref_out_w(d) <= 0) return 0;
    return 1;
}

/* ------------------------------------------------------------------------- */
/* Counter-based uniform generator for stochastic rounding.                   */
/*                                                                             */
/* The paper asks for stochastic rounding of the gradients and names neither a  */
/* generator nor the number of random bits.  Reading: a keyed hash of the      */
/* element's position, 16 bits per draw.  fmix32 is the 32-bit finalizer of    */
/* MurmurHash3 (Appleby, public domain): a bijection of 32-bit words in which  */
/* every input bit reaches every output bit.  A call with `seed` has the key   */
/*     key = fmix32(seed_lo ^ fmix32(seed_hi ^ 0x9E3779B9)),                    */
/* element idx (its NCHW linear index, below 2^31) hashes once,                */
/*     h = fmix32(idx ^ key),                                                   */
/* and the two int8 copies take disjoint halves of the word: the per-channel   */
/* copy (t = 0) draws u = (h >> 16) * 2^-16, the per-tensor copy (t = 1)       */
/* u = (h & 0xFFFF) * 2^-16, both in [0,1).                                    */
/* ------------------------------------------------------------------------- */
uint32_t daq_ref_fmix32(uint32_t h) {
    h ^= h >> 16;
    h *= UINT32_C(0x85EBCA6B);
    h ^= h >> 13;
    h *= UINT32_C(0xC2B2AE35);
    h ^= h >> 16;
    return h;
}

float daq_ref_uniform16(uint64_t seed, uint32_t tensor, uint64_t idx) {
    uint32_t lo = (uint32_t)seed, hi = (uint32_t)(seed >> 32);
    uint32_t key = daq_ref_fmix32(lo ^ daq_ref_fmix32(hi ^ UINT32_C(0x9E3779B9)));
    uint32_t h = daq_ref_fmix32((uint32_t)idx ^ key);
    uint32_t bits = tensor == 0u ? h >> 16 : h & UINT32_C(0xFFFF);
    return (float)bits * 1.52587890625e-05f; /* 2^-16, exact */
}

/* ------------------------------------------------------------------------- */
/* Symmetric uniform 8-bit quantizer, Eq. "suq" with its clamp.               */
/*   q(x) = round(127 * clamp(x, s) / s)                                       */
/* evaluated in fp32 as: inv = 127/s (one IEEE division per scale), t = x*inv, */
/* t clamped to [-127, 127] (same set of x as clamping x to [-s, s]), then     */
/* rounded.  Nearest = ties-to-even.  Stochastic = floor(t) + [frac(t) > u],    */
/* the bracket evaluated exactly.                                              */
/* ------------------------------------------------------------------------- */
int8_t daq_ref_quantize_one(float x, float s, int mode, float u) {
    if (!(s >= REF_TINY_SCALE)) return 0;
    float inv = 127.0f / s;
    float t = x * inv;
    t = fminf(fmaxf(t, -127.0f), 127.0f);
    if (mode == REF_ROUND_STOCHASTIC) {
        /* frac(t) > u, decided without rounding: t - floor(t) is not always an fp32 number (t = -2^-30 has the        */
        /* fraction 1 - 2^-30), so both sides are scaled by 2^16 and compared as doubles, where t * 2^16 is exact and */
        /* floor(t) * 2^16 + u * 2^16 is an exact integer for every 16-bit draw u.                                      */
        float f = floorf(t);
        double lhs = (double)t * 65536.0, rhs = (double)f * 65536.0 + (double)u * 65536.0;
        return (int8_t)((int)f + (lhs > rhs ? 1 : 0));
    }
    return (int8_t)(int)rintf(t);
}

/* De-quantization  x^ = q * s / 127  (text after Eq. "suq"), in fp32. */
float daq_ref_dequantize_one(int8_t q, float s) { return (float)q * (s / 127.0f); }

/* ------------------------------------------------------------------------- */
/* O1  per-channel |g|max and sigma  (Algorithm 1, "Infer |g|max and sigma").  */
/* Reading: sigma is the population standard deviation about the channel mean, */
/* accumulated in fp64, rounded once to fp32.                                  */
/* ------------------------------------------------------------------------- */
int daq_ref_channel_stats(const float* g, int N, int C, int H, int W, float* gmax, float* mean, float* sigma) {
    if (!g || !gmax || !mean || !sigma || N <= 0 || C <= 0 || H <= 0 || W <= 0) return REF_BAD_ARG;
    const size_t HW = (size_t)H * (size_t)W;
    const double M = (double)N * (double)HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        float m = 0.0f;
        double s1 = 0.0, s2 = 0.0;
        for (int n = 0; n < N; ++n) {
            const float* p = g + ((size_t)n * (size_t)C + (size_t)c) * HW;
            for (size_t i = 0; i < HW; ++i) {
                float v = p[i];
                float a = fabsf(v);
                if (a > m) m = a;
                double dv = (double)v;
                s1 += dv;
                s2 += dv * dv;
            }
        }
        double mu = s1 / M;
        double var = s2 / M - mu * mu;
        if (var < 0.0) var = 0.0;
        gmax[c] = m;
        mean[c] = (float)mu;
        sigma[c] = (float)sqrt(var);
    }
    return REF_OK;
}

/* ------------------------------------------------------------------------- */
/* O2  tail mass  P = #{ |g| > sigma } / (N*H*W)   (Algorithm 1; Eq. "judge"). */
/* Reading: the comparison is on |g| itself (no mean subtraction), as printed, */
/* in fp32.  The count is returned; P is count / M.                            */
/* ------------------------------------------------------------------------- */
int daq_ref_tail_count(const float* g, int N, int C, int H, int W, const float* sigma, uint32_t* count) {
    if (!g || !sigma || !count || N <= 0 || C <= 0 || H <= 0 || W <= 0) return REF_BAD_ARG;
    const size_t HW = (size_t)H * (size_t)W;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        uint32_t k = 0;
        const float sg = sigma[c];
        for (int n = 0; n < N; ++n) {
            const float* p = g + ((size_t)n * (size_t)C + (size_t)c) * HW;
            for (size_t i = 0; i < HW; ++i)
                if (fabsf(p[i]) > sg) ++k;
        }
        count[c] = k;
    }
    return REF_OK;
}

/* ------------------------------------------------------------------------- */
/* O3  discriminator, Eq. "judge":  Gaussian iff P > lambda, else Inverted-T.  */
/* Decided as count > lambda * M in fp64 (lambda is the fp32 argument widened) */
/* so that P == lambda falls on the Inverted-T side, as printed.               */
/* ------------------------------------------------------------------------- */
int daq_ref_classify(uint32_t count, double M, float lambda) {
    return ((double)count > (double)lambda * M) ? REF_GAUSS : REF_INVT;
}

/* ------------------------------------------------------------------------- */
/* O4  clip value.  Gaussian: s = |g|max (Eq. "gaus").  Inverted-T:            */
/*     s_t = (1 - k*A) * s_{t-1} + A * |g|max,t   (Eq. "fats"), in fp64,       */
/* rounded once to fp32.  Readings: a previous value that is not positive      */
/* (first iteration) is replaced by |g|max; a result that is not positive      */
/* (possible when 1-kA < 0) is replaced by |g|max; no upper bound is applied.  */
/* The state is overwritten with s for both classes, as the algorithm box      */
/* assigns s_{l,c,t} in both branches.                                         */
/* ------------------------------------------------------------------------- */
float daq_ref_clip_value(int cls, float gmax, float s_prev, float k, float A) {
    if (cls == REF_GAUSS) return gmax;
    float p = s_prev;
    if (!(p > 0.0f)) p = gmax;
    float s = (float)((1.0 - (double)k * (double)A) * (double)p + (double)A * (double)gmax);
    if (!(s > 0.0f)) s = gmax;
    return s;
}

/* ------------------------------------------------------------------------- */
/* Algorithm 1, first half: statistics, discriminator, clip values, then the   */
/* vectorized (per-channel) and global quantizations of the output gradient.   */
/*                                                                             */
/*  dY       fp32 [N][C][H][W]                                                 */
/*  s_state  fp32 [C] in/out, s_{l,c,t-1} -> s_{l,c,t}                         */
/*  vq, qg   int8 [N][C][H][W]   vq uses s_chan[c], qg uses s_global           */
/*  s_chan   fp32 [C];  s_global fp32 [1] = max_c |g|max,c                     */
/*  cls      u8 [C]                                                            */
/*  stats    optional fp32 [C][4] = |g|max, mean, sigma, P                     */
/*  fragile  optional u8 [C]: 1 if moving sigma by one fp32 ulp either way     */
/*           would change the class (diagnostic for parity reports)            */
/* A scale below 2^-100 is reported as 0 and gives all-zero codes.             */
/* ------------------------------------------------------------------------- */
int daq_ref_quantize_grad(const float* dY, int N, int C, int H, int W, float* s_state, float k, float A, float lambda,
                          int mode, uint64_t seed, int8_t* vq, int8_t* qg, float* s_chan, float* s_global,
                          uint8_t* cls, float* stats, uint8_t* fragile) {
    if (!dY || !s_state || !vq || !qg || !s_chan || !s_global || !cls) return REF_BAD_ARG;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0) return REF_BAD_ARG;
    if (mode != REF_ROUND_NEAREST && mode != REF_ROUND_STOCHASTIC) return REF_BAD_ARG;
    const size_t HW = (size_t)H * (size_t)W;
    const double M = (double)N * (double)HW;

    float gmax[C], mean[C], sigma[C];
    uint32_t count[C];
    int rc = daq_ref_channel_stats(dY, N, C, H, W, gmax, mean, sigma);
    if (rc) return rc;
    rc = daq_ref_tail_count(dY, N, C, H, W, sigma, count);
    if (rc) return rc;

    float sg = 0.0f;
    for (int c = 0; c < C; ++c) {
        int cl = daq_ref_classify(count[c], M, lambda);
        float s = daq_ref_clip_value(cl, gmax[c], s_state[c], k, A);
        s_state[c] = s;
        cls[c] = (uint8_t)cl;
        s_chan[c] = (s >= REF_TINY_SCALE) ? s : 0.0f;
        if (gmax[c] > sg) sg = gmax[c];
        if (stats) {
            stats[4 * c + 0] = gmax[c];
            stats[4 * c + 1] = mean[c];
            stats[4 * c + 2] = sigma[c];
            stats[4 * c + 3] = (float)((double)count[c] / M);
        }
    }
    *s_global = (sg >= REF_TINY_SCALE) ? sg : 0.0f;

    if (fragile) {
        for (int c = 0; c < C; ++c) {
            float lo = nextafterf(sigma[c], -INFINITY), hi = nextafterf(sigma[c], INFINITY);
            float two[2] = {lo, hi};
            int flip = 0;
            for (int j = 0; j < 2; ++j) {
                uint32_t k2 = 0;
                for (int n = 0; n < N; ++n) {
                    const float* p = dY + ((size_t)n * (size_t)C + (size_t)c) * HW;
                    for (size_t i = 0; i < HW; ++i)
                        if (fabsf(p[i]) > two[j]) ++k2;
                }
                if (daq_ref_classify(k2, M, lambda) != (int)cls[c]) flip = 1;
            }
            fragile[c] = (uint8_t)flip;
        }
    }

#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        const float sc = s_chan[c];
        const float sglob = *s_global;
        for (int n = 0; n < N; ++n) {
            const size_t base = ((size_t)n * (size_t)C + (size_t)c) * HW;
            for (size_t i = 0; i < HW; ++i) {
                const size_t idx = base + i;
                float u0 = 0.0f, u1 = 0.0f;
                if (mode == REF_ROUND_STOCHASTIC) {
                    u0 = daq_ref_uniform16(seed, 0u, (uint64_t)idx);
                    u1 = daq_ref_uniform16(seed, 1u, (uint64_t)idx);
                }
                vq[idx] = daq_ref_quantize_one(dY[idx], sc, mode, u0);
                qg[idx] = daq_ref_quantize_one(dY[idx], sglob, mode, u1);
            }
        }
    }
    return REF_OK;
}

/* ------------------------------------------------------------------------- */
/* Ablation schemes (experiments section, "Ablation study"): what takes the    */
/* place of the per-channel clip values of Algorithm 1 when one of its two     */
/* ingredients is switched off.  The global copy qg and s_global are the same  */
/* in every scheme.                                                            */
/*   GQ   the baseline: the whole gradient is quantized with |g|max of the     */
/*        tensor, for dW as well; s_chan[c] = max over channels of |g|max,c.   */
/*   GVQ  vectorized quantization with GQ's rule per channel: s_chan[c] =      */
/*        |g|max,c, no clipping.                                               */
/*   MCS  Magnitude-aware Clipping on the layer-wise gradient, no vectors:     */
/*        |g|max, sigma and the tail mass P of the whole tensor taken as one   */
/*        population, one class from Eq. "judge", one clip value from Eq.      */
/*        "gaus" / Eq. "fats", used for every channel.                         */
/* Readings: in GQ and GVQ the class and the statistics are still reported     */
/* per channel as Algorithm 1 computes them (they decide nothing); in MCS      */
/* every channel's row of cls / stats holds the layer's values, the previous   */
/* clip value is s_state[0], and all of s_state receives the new one.          */
/* ------------------------------------------------------------------------- */
#define REF_SCHEME_DAQ 0
#define REF_SCHEME_GQ 1
#define REF_SCHEME_GVQ 2
#define REF_SCHEME_MCS 3

/* |g|max, mean and population standard deviation of n values taken together */
int daq_ref_layer_stats(const float* g, size_t n, float* gmax, float* mean, float* sigma) {
    if (!g || !gmax || !mean || !sigma || n == 0) return REF_BAD_ARG;
    float m = 0.0f;
    double s1 = 0.0, s2 = 0.0;
    for (size_t i = 0; i < n; ++i) {
        float a = fabsf(g[i]);
        if (a > m) m = a;
        s1 += (double)g[i];
        s2 += (double)g[i] * (double)g[i];
    }
    double mu = s1 / (double)n;
    double var = s2 / (double)n - mu * mu;
    if (var < 0.0) var = 0.0;
    *gmax = m;
    *mean = (float)mu;
    *sigma = (float)sqrt(var);
    return REF_OK;
}

/* #{ |g| > sigma } over n values */
static uint32_t layer_tail_count(const float* g, size_t n, float sigma) {
    uint32_t k = 0;
    for (size_t i = 0; i < n; ++i)
        if (fabsf(g[i]) > sigma) ++k;
    return k;
}

int daq_ref_quantize_grad_scheme(const float* dY, int N, int C, int H, int W, float* s_state, float k, float A,
                                 float lambda, int mode, uint64_t seed, int scheme, int8_t* vq, int8_t* qg,
                                 float* s_chan, float* s_global, uint8_t* cls, float* stats, uint8_t* fragile) {
    if (scheme == REF_SCHEME_DAQ)
        return daq_ref_quantize_grad(dY, N, C, H, W, s_state, k, A, lambda, mode, seed, vq, qg, s_chan, s_global, cls,
                                     stats, fragile);
    if (scheme != REF_SCHEME_GQ && scheme != REF_SCHEME_GVQ && scheme != REF_SCHEME_MCS) return REF_BAD_ARG;
    if (!dY || !s_state || !vq || !qg || !s_chan || !s_global || !cls) return REF_BAD_ARG;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0) return REF_BAD_ARG;
    if (mode != REF_ROUND_NEAREST && mode != REF_ROUND_STOCHASTIC) return REF_BAD_ARG;
    const size_t HW = (size_t)H * (size_t)W;
    const size_t total = (size_t)N * (size_t)C * HW;
    const double M = (double)N * (double)HW;

    float gmax[C], mean[C], sigma[C];
    uint32_t count[C];
    int rc = daq_ref_channel_stats(dY, N, C, H, W, gmax, mean, sigma);
    if (rc) return rc;
    rc = daq_ref_tail_count(dY, N, C, H, W, sigma, count);
    if (rc) return rc;
    float sg = 0.0f;
    for (int c = 0; c < C; ++c)
        if (gmax[c] > sg) sg = gmax[c];
    *s_global = (sg >= REF_TINY_SCALE) ? sg : 0.0f;

    if (scheme == REF_SCHEME_MCS) {
        float gm_l, mu_l, sig_l;
        rc = daq_ref_layer_stats(dY, total, &gm_l, &mu_l, &sig_l);
        if (rc) return rc;
        const uint32_t cnt = layer_tail_count(dY, total, sig_l);
        const int cl = daq_ref_classify(cnt, (double)total, lambda);
        const float s = daq_ref_clip_value(cl, gm_l, s_state[0], k, A);
        int flip = 0;
        if (fragile) {
            if (daq_ref_classify(layer_tail_count(dY, total, nextafterf(sig_l, -INFINITY)), (double)total, lambda) != cl) flip = 1;
            if (daq_ref_classify(layer_tail_count(dY, total, nextafterf(sig_l, INFINITY)), (double)total, lambda) != cl) flip = 1;
        }
        for (int c = 0; c < C; ++c) {
            s_state[c] = s;
            s_chan[c] = (s >= REF_TINY_SCALE) ? s : 0.0f;
            cls[c] = (uint8_t)cl;
            if (fragile) fragile[c] = (uint8_t)flip;
            if (stats) {
                stats[4 * c + 0] = gm_l;
                stats[4 * c + 1] = mu_l;
                stats[4 * c + 2] = sig_l;
                stats[4 * c + 3] = (float)((double)cnt / (double)total);
            }
        }
    } else {
        for (int c = 0; c < C; ++c) {
            const float s = (scheme == REF_SCHEME_GQ) ? sg : gmax[c];
            s_state[c] = s;
            s_chan[c] = (s >= REF_TINY_SCALE) ? s : 0.0f;
            cls[c] = (uint8_t)daq_ref_classify(count[c], M, lambda);
            if (stats) {
                stats[4 * c + 0] = gmax[c];
                stats[4 * c + 1] = mean[c];
                stats[4 * c + 2] = sigma[c];
                stats[4 * c + 3] = (float)((double)count[c] / M);
            }
            if (fragile) {
                const float two[2] = {nextafterf(sigma[c], -INFINITY), nextafterf(sigma[c], INFINITY)};
                int flip = 0;
                for (int j = 0; j < 2; ++j) {
                    uint32_t k2 = 0;
                    for (int n = 0; n < N; ++n) {
                        const float* p = dY + ((size_t)n * (size_t)C + (size_t)c) * HW;
                        for (size_t i = 0; i < HW; ++i)
                            if (fabsf(p[i]) > two[j]) ++k2;
                    }
                    if (daq_ref_classify(k2, M, lambda) != (int)cls[c]) flip = 1;
                }
                fragile[c] = (uint8_t)flip;
            }
        }
    }

#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        for (int n = 0; n < N; ++n) {
            const size_t base = ((size_t)n * (size_t)C + (size_t)c) * HW;
            for (size_t i = 0; i < HW; ++i) {
                const size_t idx = base + i;
                float u0 = 0.0f, u1 = 0.0f;
                if (mode == REF_ROUND_STOCHASTIC) {
                    u0 = daq_ref_uniform16(seed, 0u, (uint64_t)idx);
                    u1 = daq_ref_uniform16(seed, 1u, (uint64_t)idx);
                }
                vq[idx] = daq_ref_quantize_one(dY[idx], s_chan[c], mode, u0);
                qg[idx] = daq_ref_quantize_one(dY[idx], *s_global, mode, u1);
            }
        }
    }
    return REF_OK;
}

/* ------------------------------------------------------------------------- */
/* Per-tensor ("global") quantization used in the forward pass for X and W:    */
/* s = max|x| (reading: the paper defers the forward rule to earlier work and  */
/* calls it global quantization; max-abs is taken), nearest rounding.          */
/* ------------------------------------------------------------------------- */
/* ------------------------------------------------------------------------- */
/* The objective of the Magnitude-aware Clipping Strategy, Eq. "e", minimised  */
/* by search: for channel c and candidate s_j = |g|max_c * (j / J), j = 1..J,  */
/*   E_c(s_j) = (1/M) sum |g - g^| * exp(alpha |g|),  g^ = Q(g, s_j) * s_j/127 */
/* (Q and the de-quantization as above, nearest rounding; difference, weight   */
/* and sum in fp64, elements in NCHW order).  best_j = first j of the smallest */
/* error, best_s = s_{best_j}.                                                 */
/* ------------------------------------------------------------------------- */
int daq_ref_clip_search(const float* g, int N, int C, int H, int W, float alpha, int J, double* err, float* best_s,
                        int32_t* best_j) {
    if (!g || !err || !best_s || !best_j || N <= 0 || C <= 0 || H <= 0 || W <= 0 || J < 1 || !(alpha >= 0.0f)) return REF_BAD_ARG;
    const size_t HW = (size_t)H * W;
    const double M = (double)N * (double)HW;
#pragma omp parallel for schedule(dynamic, 1)
    for (int c = 0; c < C; ++c) {
        float gmax = 0.0f;
        for (int n = 0; n < N; ++n)
            for (size_t i = 0; i < HW; ++i) gmax = fmaxf(gmax, fabsf(g[((size_t)n * C + c) * HW + i]));
        int arg = 0;
        for (int j = 1; j <= J; ++j) {
            const float s = gmax * ((float)j / (float)J);
            double sum = 0.0;
            for (int n = 0; n < N; ++n)
                for (size_t i = 0; i < HW; ++i) {
                    const float x = g[((size_t)n * C + c) * HW + i];
                    const float gh = daq_ref_dequantize_one(daq_ref_quantize_one(x, s, REF_ROUND_NEAREST, 0.0f), s >= REF_TINY_SCALE ? s : 0.0f);
                    sum += fabs((double)x - (double)gh) * exp((double)alpha * (double)fabsf(x));
                }
            err[(size_t)c * J + (j - 1)] = sum / M;
            if (j > 1 && err[(size_t)c * J + (j - 1)] < err[(size_t)c * J + arg]) arg = j - 1;
        }
        best_j[c] = arg + 1;
        best_s[c] = gmax * ((float)(arg + 1) / (float)J);
    }
    return REF_OK;
}

int daq_ref_quantize_tensor(const float* x, size_t n, int8_t* q, float* s_out) {
    if (!x || !q || !s_out) return REF_BAD_ARG;
    float m = 0.0f;
    for (size_t i = 0; i < n; ++i) {
        float a = fabsf(x[i]);
        if (a > m) m = a;
    }
    float s = (m >= REF_TINY_SCALE) ? m : 0.0f;
    *s_out = s;
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) q[i] = daq_ref_quantize_one(x[i], s, REF_ROUND_NEAREST, 0.0f);
    return REF_OK;
}

static int32_t wrap32(int64_t a, int* overflow) {
    if (a > (int64_t)INT32_MAX || a < (int64_t)INT32_MIN) *overflow = 1;
    return (int32_t)(uint32_t)(uint64_t)a;
}

/* ------------------------------------------------------------------------- */
/* Forward integer convolution  acc[n,co,ho,wo] = sum qX * qW  over            */
/* (ci within the group, kh, kw) with zero padding.                            */
/* ------------------------------------------------------------------------- */
int daq_ref_conv_fwd_acc(const ref_conv_desc* d, const int8_t* qX, const int8_t* qW, int32_t* acc, int* overflow) {
    if (!desc_ok(d) || !qX || !qW || !acc || !overflow) return REF_BAD_ARG;
    const int Ho = daq_ref_out_h(d), Wo = daq_ref_out_w(d);
    const int cig = d->Cin / d->groups, cog = d->Cout / d->groups;
    int ovf = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : ovf)
    for (int n = 0; n < d->N; ++n)
        for (int co = 0; co < d->Cout; ++co) {
            const int g = co / cog;
            for (int ho = 0; ho < Ho; ++ho)
                for (int wo = 0; wo < Wo; ++wo) {
                    int64_t a = 0;
                    for (int cl = 0; cl < cig; ++cl) {
                        const int ci = g * cig + cl;
                        for (int kh = 0; kh < d->kH; ++kh) {
                            const int h = ho * d->strideH + kh * d->dilH - d->padH;
                            if (h < 0 || h >= d->Hin) continue;
                            for (int kw = 0; kw < d->kW; ++kw) {
                                const int w = wo * d->strideW + kw * d->dilW - d->padW;
                                if (w < 0 || w >= d->Win) continue;
                                const int8_t xv = qX[(((size_t)n * d->Cin + ci) * d->Hin + h) * d->Win + w];
                                const int8_t wv = qW[(((size_t)co * cig + cl) * d->kH + kh) * d->kW + kw];
                                a += (int64_t)xv * (int64_t)wv;
                            }
                        }
                    }
                    int o = 0;
                    acc[(((size_t)n * d->Cout + co) * Ho + ho) * Wo + wo] = wrap32(a, &o);
                    ovf |= o;
                }
        }
    *overflow = ovf;
    return REF_OK;
}

/* ------------------------------------------------------------------------- */
/* Data gradient, Eq. "gx":  acc[n,ci,h,w] = sum over (co in the group, kh,kw) */
/* of qG[n,co,ho,wo] * qW[co,ci,kh,kw] where ho*stride + kh*dil - pad == h     */
/* (and likewise for w) with ho, wo integral and inside the output.            */
/* ------------------------------------------------------------------------- */
int daq_ref_conv_bwd_data_acc(const ref_conv_desc* d, const int8_t* qG, const int8_t* qW, int32_t* acc,
                              int* overflow) {
    if (!desc_ok(d) || !qG || !qW || !acc || !overflow) return REF_BAD_ARG;
    const int Ho = daq_ref_out_h(d), Wo = daq_ref_out_w(d);
    const int cig = d->Cin / d->groups, cog = d->Cout / d->groups;
    int ovf = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : ovf)
    for (int n = 0; n < d->N; ++n)
        for (int ci = 0; ci < d->Cin; ++ci) {
            const int g = ci / cig, cl = ci % cig;
            for (int h = 0; h < d->Hin; ++h)
                for (int w = 0; w < d->Win; ++w) {
                    int64_t a = 0;
                    for (int col = 0; col < cog; ++col) {
                        const int co = g * cog + col;
                        for (int kh = 0; kh < d->kH; ++kh) {
                            const int hn = h + d->padH - kh * d->dilH;
                            if (hn < 0 || hn % d->strideH) continue;
                            const int ho = hn / d->strideH;
                            if (ho >= Ho) continue;
                            for (int kw = 0; kw < d->kW; ++kw) {
                                const int wn = w + d->padW - kw * d->dilW;
                                if (wn < 0 || wn % d->strideW) continue;
                                const int wo = wn / d->strideW;
                                if (wo >= Wo) continue;
                                const int8_t gv = qG[(((size_t)n * d->Cout + co) * Ho + ho) * Wo + wo];
                                const int8_t wv = qW[(((size_t)co * cig + cl) * d->kH + kh) * d->kW + kw];
                                a += (int64_t)gv * (int64_t)wv;
                            }
                        }
                    }
                    int o = 0;
                    acc[(((size_t)n * d->Cin + ci) * d->Hin + h) * d->Win + w] = wrap32(a, &o);
                    ovf |= o;
                }
        }
    *overflow = ovf;
    return REF_OK;
}

/* ------------------------------------------------------------------------- */
/* Filter gradient, Eq. "gw":  acc[co,cl,kh,kw] = sum over (n,ho,wo) of        */
/* qX[n,ci,ho*stride+kh*dil-pad, wo*stride+kw*dil-pad] * qG[n,co,ho,wo],       */
/* zero outside the input.                                                     */
/* ------------------------------------------------------------------------- */
int daq_ref_conv_bwd_filter_acc(const ref_conv_desc* d, const int8_t* qX, const int8_t* qG, int32_t* acc,
                                int* overflow) {
    if (!desc_ok(d) || !qX || !qG || !acc || !overflow) return REF_BAD_ARG;
    const int Ho = daq_ref_out_h(d), Wo = daq_ref_out_w(d);
    const int cig = d->Cin / d->groups, cog = d->Cout / d->groups;
    int ovf = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : ovf)
    for (int co = 0; co < d->Cout; ++co)
        for (int cl = 0; cl < cig; ++cl) {
            const int g = co / cog;
            const int ci = g * cig + cl;
            for (int kh = 0; kh < d->kH; ++kh)
                for (int kw = 0; kw < d->kW; ++kw) {
                    int64_t a = 0;
                    for (int n = 0; n < d->N; ++n)
                        for (int ho = 0; ho < Ho; ++ho) {
                            const int h = ho * d->strideH + kh * d->dilH - d->padH;
                            if (h < 0 || h >= d->Hin) continue;
                            for (int wo = 0; wo < Wo; ++wo) {
                                const int w = wo * d->strideW + kw * d->dilW - d->padW;
                                if (w < 0 || w >= d->Win) continue;
                                const int8_t xv = qX[(((size_t)n * d->Cin + ci) * d->Hin + h) * d->Win + w];
                                const int8_t gv = qG[(((size_t)n * d->Cout + co) * Ho + ho) * Wo + wo];
                                a += (int64_t)xv * (int64_t)gv;
                            }
                        }
                    int o = 0;
                    acc[(((size_t)co * cig + cl) * d->kH + kh) * d->kW + kw] = wrap32(a, &o);
                    ovf |= o;
                }
        }
    *overflow = ovf;
    return REF_OK;
}

/* ------------------------------------------------------------------------- */
/* Single elements of the two gradients, for checks at sizes where the whole    */
/* tensor is too much for the loops above.  Same definitions (Eq. "gx", "gw"),  */
/* one output per index: idx[i] is the linear NCHW index into G_X, or the       */
/* linear [Cout][Cin/groups][kH][kW] index into G_W.  Values wrap to int32.     */
/* ------------------------------------------------------------------------- */
int daq_ref_conv_bwd_data_acc_at(const ref_conv_desc* d, const int8_t* qG, const int8_t* qW, const int64_t* idx,
                                 int64_t count, int32_t* out) {
    if (!desc_ok(d) || !qG || !qW || !idx || !out || count < 0) return REF_BAD_ARG;
    const int Ho = daq_ref_out_h(d), Wo = daq_ref_out_w(d);
    const int cig = d->Cin / d->groups, cog = d->Cout / d->groups;
    const int64_t total = (int64_t)d->N * d->Cin * d->Hin * d->Win;
    for (int64_t i = 0; i < count; ++i)
        if (idx[i] < 0 || idx[i] >= total) return REF_BAD_ARG;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t i = 0; i < count; ++i) {
        int64_t r = idx[i];
        const int w = (int)(r % d->Win); r /= d->Win;
        const int h = (int)(r % d->Hin); r /= d->Hin;
        const int ci = (int)(r % d->Cin);
        const int n = (int)(r / d->Cin);
        const int g = ci / cig, cl = ci % cig;
        int64_t a = 0;
        for (int col = 0; col < cog; ++col) {
            const int co = g * cog + col;
            for (int kh = 0; kh < d->kH; ++kh) {
                /* the output row that tap kh of this input row contributed to in the forward pass, if any */
                const int hn = h + d->padH - kh * d->dilH;
                if (hn < 0 || hn % d->strideH || hn / d->strideH >= Ho) continue;
                for (int kw = 0; kw < d->kW; ++kw) {
                    const int wn = w + d->padW - kw * d->dilW;
                    if (wn < 0 || wn % d->strideW || wn / d->strideW >= Wo) continue;
                    const int8_t gv = qG[(((size_t)n * d->Cout + co) * Ho + hn / d->strideH) * Wo + wn / d->strideW];
                    const int8_t wv = qW[(((size_t)co * cig + cl) * d->kH + kh) * d->kW + kw];
                    a += (int64_t)gv * (int64_t)wv;
                }
            }
        }
        int o = 0;
        out[i] = wrap32(a, &o);
    }
    return REF_OK;
}

int daq_ref_conv_bwd_filter_acc_at(const ref_conv_desc* d, const int8_t* qX, const int8_t* qG, const int64_t* idx,
                                   int64_t count, int32_t* out) {
    if (!desc_ok(d) || !qX || !qG || !idx || !out || count < 0) return REF_BAD_ARG;
    const int Ho = daq_ref_out_h(d), Wo = daq_ref_out_w(d);
    const int cig = d->Cin / d->groups, cog = d->Cout / d->groups;
    const int64_t total = (int64_t)d->Cout * cig * d->kH * d->kW;
    for (int64_t i = 0; i < count; ++i)
        if (idx[i] < 0 || idx[i] >= total) return REF_BAD_ARG;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < count; ++i) {
        int64_t r = idx[i];
        const int kw = (int)(r % d->kW); r /= d->kW;
        const int kh = (int)(r % d->kH); r /= d->kH;
        const int cl = (int)(r % cig);
        const int co = (int)(r / cig);
        const int ci = (co / cog) * cig + cl;
        int64_t a = 0;
        for (int n = 0; n < d->N; ++n)
            for (int ho = 0; ho < Ho; ++ho) {
                const int h = ho * d->strideH + kh * d->dilH - d->padH;
                if (h < 0 || h >= d->Hin) continue;
                for (int wo = 0; wo < Wo; ++wo) {
                    const int w = wo * d->strideW + kw * d->dilW - d->padW;
                    if (w < 0 || w >= d->Win) continue;
                    a += (int64_t)qX[(((size_t)n * d->Cin + ci) * d->Hin + h) * d->Win + w] *
                         (int64_t)qG[(((size_t)n * d->Cout + co) * Ho + ho) * Wo + wo];
                }
            }
        int o = 0;
        out[i] = wrap32(a, &o);
    }
    return REF_OK;
}

/* Forward accumulators at single positions: idx[i] is the linear NCHW index into Y
 * (the integer convolution of daq_ref_conv_fwd_acc, one output per index). */
int daq_ref_conv_fwd_acc_at(const ref_conv_desc* d, const int8_t* qX, const int8_t* qW, const int64_t* idx,
                            int64_t count, int32_t* out) {
    if (!desc_ok(d) || !qX || !qW || !idx || !out || count < 0) return REF_BAD_ARG;
    const int Ho = daq_ref_out_h(d), Wo = daq_ref_out_w(d);
    const int cig = d->Cin / d->groups, cog = d->Cout / d->groups;
    const int64_t total = (int64_t)d->N * d->Cout * Ho * Wo;
    for (int64_t i = 0; i < count; ++i)
        if (idx[i] < 0 || idx[i] >= total) return REF_BAD_ARG;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t i = 0; i < count; ++i) {
        int64_t r = idx[i];
        const int wo = (int)(r % Wo); r /= Wo;
        const int ho = (int)(r % Ho); r /= Ho;
        const int co = (int)(r % d->Cout);
        const int n = (int)(r / d->Cout);
        const int g = co / cog;
        int64_t a = 0;
        for (int cl = 0; cl < cig; ++cl) {
            const int ci = g * cig + cl;
            for (int kh = 0; kh < d->kH; ++kh) {
                const int h = ho * d->strideH + kh * d->dilH - d->padH;
                if (h < 0 || h >= d->Hin) continue;
                for (int kw = 0; kw < d->kW; ++kw) {
                    const int w = wo * d->strideW + kw * d->dilW - d->padW;
                    if (w < 0 || w >= d->Win) continue;
                    a += (int64_t)qX[(((size_t)n * d->Cin + ci) * d->Hin + h) * d->Win + w] *
                         (int64_t)qW[(((size_t)co * cig + cl) * d->kH + kh) * d->kW + kw];
                }
            }
        }
        int o = 0;
        out[i] = wrap32(a, &o);
    }
    return REF_OK;
}

/* ------------------------------------------------------------------------- */
/* De-quantization of an accumulator: acc * (s_a/127) * (s_b/127), evaluated   */
/* in fp32 as  (float)acc * ((s_a/127) * (s_b/127)).                           */
/* ------------------------------------------------------------------------- */
static float dq2(int32_t acc, float sa, float sb) { return (float)acc * ((sa / 127.0f) * (sb / 127.0f)); }

/* The same product for a list of accumulators: out[i] = acc[i] * (s_a/127) * (s_b[i]/127).  s_b carries one
 * scale per element, so that the caller can hand over the per-tensor scale of the data gradient or the clip
 * value of each element's output channel (the vectorized de-quantization of the filter gradient). */
int daq_ref_dequantize_acc(const int32_t* acc, int64_t count, float s_a, const float* s_b, float* out) {
    if (!acc || !s_b || !out || count < 0) return REF_BAD_ARG;
    for (int64_t i = 0; i < count; ++i) out[i] = dq2(acc[i], s_a, s_b[i]);
    return REF_OK;
}

/* Forward pass of one layer: quantize X and W per tensor, integer convolution,
 * Y = acc * s_x/127 * s_w/127.  qX, qW, s_x, s_w are what the backward pass
 * of Algorithm 1 requires as saved inputs. */
int daq_ref_conv_fwd_int8(const ref_conv_desc* d, const float* X, const float* Wt, int8_t* qX, int8_t* qW, float* s_x,
                          float* s_w, float* Y, int32_t* acc_out, int* overflow) {
    if (!desc_ok(d) || !X || !Wt || !qX || !qW || !s_x || !s_w || !Y || !overflow) return REF_BAD_ARG;
    const int Ho = daq_ref_out_h(d), Wo = daq_ref_out_w(d);
    const size_t nx = (size_t)d->N * d->Cin * d->Hin * d->Win;
    const size_t nw = (size_t)d->Cout * (d->Cin / d->groups) * d->kH * d->kW;
    const size_t ny = (size_t)d->N * d->Cout * Ho * Wo;
    int rc = daq_ref_quantize_tensor(X, nx, qX, s_x);
    if (rc) return rc;
    rc = daq_ref_quantize_tensor(Wt, nw, qW, s_w);
    if (rc) return rc;
    int32_t* acc = acc_out;
    int32_t* tmp = NULL;
    if (!acc) {
        tmp = (int32_t*)malloc(ny * sizeof(int32_t));
        if (!tmp) return REF_BAD_ARG;
        acc = tmp;
    }
    rc = daq_ref_conv_fwd_acc(d, qX, qW, acc, overflow);
    if (!rc)
        for (size_t i = 0; i < ny; ++i) Y[i] = dq2(acc[i], *s_x, *s_w);
    free(tmp);
    return rc;
}

/* Algorithm 1: q(G_X) = q(G) (transposed conv) q(W), then global de-quantization
 * with the scales of its two operands, s_global and s_w.  (The algorithm box
 * prints s_X here and s_W for G_W; the operands of each product, and the
 * per-channel de-quantization formula in the text, fix the pairing used.) */
int daq_ref_conv_bwd_data_int8(const ref_conv_desc* d, const int8_t* qG, float s_global, const int8_t* qW, float s_w,
                               float* dX, int32_t* acc_out, int* overflow) {
    if (!desc_ok(d) || !dX || !acc_out) return REF_BAD_ARG;
    int rc = daq_ref_conv_bwd_data_acc(d, qG, qW, acc_out, overflow);
    if (rc) return rc;
    const size_t nx = (size_t)d->N * d->Cin * d->Hin * d->Win;
    for (size_t i = 0; i < nx; ++i) dX[i] = dq2(acc_out[i], s_w, s_global);
    return REF_OK;
}

/* Depthwise variant (the MobileNetV2 paragraph's layers, groups = Cin = Cout): input-gradient channel c is
 * a function of output-gradient channel c alone, so the per-channel copy and its clip values can serve for
 * G_X too:  G_X[n,c] = (sum over taps of vq[n,c] * qW[c]) * s_w/127 * s_chan[c]/127.
 * An option beside Algorithm 1, which quantizes G with the global |g|max for G_X. */
int daq_ref_conv_bwd_data_int8_chan(const ref_conv_desc* d, const int8_t* vq, const float* s_chan, const int8_t* qW,
                                    float s_w, float* dX, int32_t* acc_out, int* overflow) {
    if (!desc_ok(d) || !dX || !acc_out || !s_chan) return REF_BAD_ARG;
    if (d->groups != d->Cin || d->groups != d->Cout) return REF_BAD_ARG;
    int rc = daq_ref_conv_bwd_data_acc(d, vq, qW, acc_out, overflow);
    if (rc) return rc;
    const size_t plane = (size_t)d->Hin * d->Win;
    for (int n = 0; n < d->N; ++n)
        for (int c = 0; c < d->Cin; ++c)
            for (size_t i = 0; i < plane; ++i) {
                const size_t at = ((size_t)n * d->Cin + c) * plane + i;
                dX[at] = dq2(acc_out[at], s_w, s_chan[c]);
            }
    return REF_OK;
}

/* Algorithm 1: q(G_W) = q(X') (dilated conv) vq(G'), then vectorized
 * de-quantization  G_W[co] = acc[co] * s_x/127 * s_chan[co]/127. */
int daq_ref_conv_bwd_filter_int8(const ref_conv_desc* d, const int8_t* qX, float s_x, const int8_t* vq,
                                 const float* s_chan, float* dW, int32_t* acc_out, int* overflow) {
    if (!desc_ok(d) || !dW || !acc_out || !s_chan) return REF_BAD_ARG;
    int rc = daq_ref_conv_bwd_filter_acc(d, qX, vq, acc_out, overflow);
    if (rc) return rc;
    const size_t per = (size_t)(d->Cin / d->groups) * d->kH * d->kW;
    for (int co = 0; co < d->Cout; ++co)
        for (size_t i = 0; i < per; ++i) dW[co * per + i] = dq2(acc_out[co * per + i], s_x, s_chan[co]);
    return REF_OK;
}


/* ========================================================================= */
/* 3-D convolution (the video-classification experiment: the depth axis is    */
/* treated like height and width).  Tensors: X in (N, Cin, Din, Hin, Win),     */
/* W in (Cout, Cin/groups, kD, kH, kW), Y and G in (N, Cout, Do, Ho, Wo).      */
/* Same definitions as the 2-D routines with one more spatial axis; the        */
/* quantizer needs no 3-D form: its statistics run over all of (n, d, h, w),   */
/* which is the 2-D routine on the tensor viewed as (N, C, D*H, W).            */
/* ========================================================================= */
typedef struct {
    int N, Cin, Din, Hin, Win;
    int Cout, kD, kH, kW;
    int strideD, strideH, strideW;
    int padD, padH, padW;
    int dilD, dilH, dilW;
    int groups;
} ref_conv3d_desc;

int daq_ref_out_d3(const ref_conv3d_desc* d) { return out_dim(d->Din, d->padD, d->dilD, d->kD, d->strideD); }
int daq_ref_out_h3(const ref_conv3d_desc* d) { return out_dim(d->Hin, d->padH, d->dilH, d->kH, d->strideH); }
int daq_ref_out_w3(const ref_conv3d_desc* d) { return out_dim(d->Win, d->padW, d->dilW, d->kW, d->strideW); }

static int desc3_ok(const ref_conv3d_desc* d) {
    if (!d) return 0;
    if (d->N <= 0 || d->Cin <= 0 || d->Din <= 0 || d->Hin <= 0 || d->Win <= 0 || d->Cout <= 0) return 0;
    if (d->kD <= 0 || d->kH <= 0 || d->kW <= 0 || d->strideD <= 0 || d->strideH <= 0 || d->strideW <= 0) return 0;
    if (d->padD < 0 || d->padH < 0 || d->padW < 0 || d->dilD <= 0 || d->dilH <= 0 || d->dilW <= 0 || d->groups <= 0) return 0;
    if (d->Cin % d->groups || d->Cout % d->groups) return 0;
    if (daq_ref_out_d3(d) <= 0 || daq_ref_out_h3(d) <= 0 || daq_ref_out_w3(d) <= 0) return 0;
    return 1;
}

/* forward: acc[n,co,do,ho,wo] = sum over (ci in the group, kd, kh, kw) of qX[n,ci,do*s+kd*dil-p,...] * qW[co,cl,kd,kh,kw] */
int daq_ref_conv3d_fwd_acc(const ref_conv3d_desc* d, const int8_t* qX, const int8_t* qW, int32_t* acc, int* overflow) {
    if (!desc3_ok(d) || !qX || !qW || !acc || !overflow) return REF_BAD_ARG;
    const int Do = daq_ref_out_d3(d), Ho = daq_ref_out_h3(d), Wo = daq_ref_out_w3(d);
    const int cig = d->Cin / d->groups, cog = d->Cout / d->groups;
    int ovf = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : ovf)
    for (int n = 0; n < d->N; ++n)
        for (int co = 0; co < d->Cout; ++co) {
            const int g = co / cog;
            for (int od = 0; od < Do; ++od)
                for (int ho = 0; ho < Ho; ++ho)
                    for (int wo = 0; wo < Wo; ++wo) {
                        int64_t a = 0;
                        for (int cl = 0; cl < cig; ++cl) {
                            const int ci = g * cig + cl;
                            for (int kd = 0; kd < d->kD; ++kd) {
                                const int z = od * d->strideD + kd * d->dilD - d->padD;
                                if (z < 0 || z >= d->Din) continue;
                                for (int kh = 0; kh < d->kH; ++kh) {
                                    const int h = ho * d->strideH + kh * d->dilH - d->padH;
                                    if (h < 0 || h >= d->Hin) continue;
                                    for (int kw = 0; kw < d->kW; ++kw) {
                                        const int w = wo * d->strideW + kw * d->dilW - d->padW;
                                        if (w < 0 || w >= d->Win) continue;
                                        a += (int64_t)qX[((((size_t)n * d->Cin + ci) * d->Din + z) * d->Hin + h) * d->Win + w] *
                                             (int64_t)qW[((((size_t)co * cig + cl) * d->kD + kd) * d->kH + kh) * d->kW + kw];
                                    }
                                }
                            }
                        }
                        int o = 0;
                        acc[((((size_t)n * d->Cout + co) * Do + od) * Ho + ho) * Wo + wo] = wrap32(a, &o);
                        ovf |= o;
                    }
        }
    *overflow = ovf;
    return REF_OK;
}

/* data gradient: acc[n,ci,z,h,w] = sum over (co in the group, kd, kh, kw) of qG[n,co,od,ho,wo] * qW[co,cl,kd,kh,kw]
 * where od*stride + kd*dil - pad == z with od integral and inside the output (same for the other two axes) */
int daq_ref_conv3d_bwd_data_acc(const ref_conv3d_desc* d, const int8_t* qG, const int8_t* qW, int32_t* acc, int* overflow) {
    if (!desc3_ok(d) || !qG || !qW || !acc || !overflow) return REF_BAD_ARG;
    const int Do = daq_ref_out_d3(d), Ho = daq_ref_out_h3(d), Wo = daq_ref_out_w3(d);
    const int cig = d->Cin / d->groups, cog = d->Cout / d->groups;
    int ovf = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : ovf)
    for (int n = 0; n < d->N; ++n)
        for (int ci = 0; ci < d->Cin; ++ci) {
            const int g = ci / cig, cl = ci % cig;
            for (int z = 0; z < d->Din; ++z)
                for (int h = 0; h < d->Hin; ++h)
                    for (int w = 0; w < d->Win; ++w) {
                        int64_t a = 0;
                        for (int col = 0; col < cog; ++col) {
                            const int co = g * cog + col;
                            for (int kd = 0; kd < d->kD; ++kd) {
                                const int zn = z + d->padD - kd * d->dilD;
                                if (zn < 0 || zn % d->strideD || zn / d->strideD >= Do) continue;
                                for (int kh = 0; kh < d->kH; ++kh) {
                                    const int hn = h + d->padH - kh * d->dilH;
                                    if (hn < 0 || hn % d->strideH || hn / d->strideH >= Ho) continue;
                                    for (int kw = 0; kw < d->kW; ++kw) {
                                        const int wn = w + d->padW - kw * d->dilW;
                                        if (wn < 0 || wn % d->strideW || wn / d->strideW >= Wo) continue;
                                        a += (int64_t)qG[((((size_t)n * d->Cout + co) * Do + zn / d->strideD) * Ho + hn / d->strideH) * Wo + wn / d->strideW] *
                                             (int64_t)qW[((((size_t)co * cig + cl) * d->kD + kd) * d->kH + kh) * d->kW + kw];
                                    }
                                }
                            }
                        }
                        int o = 0;
                        acc[((((size_t)n * d->Cin + ci) * d->Din + z) * d->Hin + h) * d->Win + w] = wrap32(a, &o);
                        ovf |= o;
                    }
        }
    *overflow = ovf;
    return REF_OK;
}

/* filter gradient: acc[co,cl,kd,kh,kw] = sum over (n, od, ho, wo) of qX[n,ci,od*s+kd*dil-p,...] * qG[n,co,od,ho,wo] */
int daq_ref_conv3d_bwd_filter_acc(const ref_conv3d_desc* d, const int8_t* qX, const int8_t* qG, int32_t* acc, int* overflow) {
    if (!desc3_ok(d) || !qX || !qG || !acc || !overflow) return REF_BAD_ARG;
    const int Do = daq_ref_out_d3(d), Ho = daq_ref_out_h3(d), Wo = daq_ref_out_w3(d);
    const int cig = d->Cin / d->groups, cog = d->Cout / d->groups;
    int ovf = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : ovf)
    for (int co = 0; co < d->Cout; ++co)
        for (int cl = 0; cl < cig; ++cl) {
            const int ci = (co / cog) * cig + cl;
            for (int kd = 0; kd < d->kD; ++kd)
                for (int kh = 0; kh < d->kH; ++kh)
                    for (int kw = 0; kw < d->kW; ++kw) {
                        int64_t a = 0;
                        for (int n = 0; n < d->N; ++n)
                            for (int od = 0; od < Do; ++od) {
                                const int z = od * d->strideD + kd * d->dilD - d->padD;
                                if (z < 0 || z >= d->Din) continue;
                                for (int ho = 0; ho < Ho; ++ho) {
                                    const int h = ho * d->strideH + kh * d->dilH - d->padH;
                                    if (h < 0 || h >= d->Hin) continue;
                                    for (int wo = 0; wo < Wo; ++wo) {
                                        const int w = wo * d->strideW + kw * d->dilW - d->padW;
                                        if (w < 0 || w >= d->Win) continue;
                                        a += (int64_t)qX[((((size_t)n * d->Cin + ci) * d->Din + z) * d->Hin + h) * d->Win + w] *
                                             (int64_t)qG[((((size_t)n * d->Cout + co) * Do + od) * Ho + ho) * Wo + wo];
                                    }
                                }
                            }
                        int o = 0;
                        acc[((((size_t)co * cig + cl) * d->kD + kd) * d->kH + kh) * d->kW + kw] = wrap32(a, &o);
                        ovf |= o;
                    }
        }
    *overflow = ovf;
    return REF_OK;
}

/* The three layer routines: the 2-D ones with the 3-D products (same quantizers, same de-quantization pairing). */
int daq_ref_conv3d_fwd_int8(const ref_conv3d_desc* d, const float* X, const float* Wt, int8_t* qX, int8_t* qW, float* s_x,
                            float* s_w, float* Y, int32_t* acc, int* overflow) {
    if (!desc3_ok(d) || !X || !Wt || !qX || !qW || !s_x || !s_w || !Y || !acc || !overflow) return REF_BAD_ARG;
    const size_t nx = (size_t)d->N * d->Cin * d->Din * d->Hin * d->Win;
    const size_t nw = (size_t)d->Cout * (d->Cin / d->groups) * d->kD * d->kH * d->kW;
    const size_t ny = (size_t)d->N * d->Cout * daq_ref_out_d3(d) * daq_ref_out_h3(d) * daq_ref_out_w3(d);
    int rc = daq_ref_quantize_tensor(X, nx, qX, s_x);
    if (rc) return rc;
    rc = daq_ref_quantize_tensor(Wt, nw, qW, s_w);
    if (rc) return rc;
    rc = daq_ref_conv3d_fwd_acc(d, qX, qW, acc, overflow);
    if (!rc)
        for (size_t i = 0; i < ny; ++i) Y[i] = dq2(acc[i], *s_x, *s_w);
    return rc;
}

int daq_ref_conv3d_bwd_data_int8(const ref_conv3d_desc* d, const int8_t* qG, float s_global, const int8_t* qW, float s_w,
                                 float* dX, int32_t* acc, int* overflow) {
    if (!desc3_ok(d) || !dX || !acc) return REF_BAD_ARG;
    int rc = daq_ref_conv3d_bwd_data_acc(d, qG, qW, acc, overflow);
    if (rc) return rc;
    const size_t nx = (size_t)d->N * d->Cin * d->Din * d->Hin * d->Win;
    for (size_t i = 0; i < nx; ++i) dX[i] = dq2(acc[i], s_w, s_global);
    return REF_OK;
}

int daq_ref_conv3d_bwd_filter_int8(const ref_conv3d_desc* d, const int8_t* qX, float s_x, const int8_t* vq, const float* s_chan,
                                   float* dW, int32_t* acc, int* overflow) {
    if (!desc3_ok(d) || !dW || !acc || !s_chan) return REF_BAD_ARG;
    int rc = daq_ref_conv3d_bwd_filter_acc(d, qX, vq, acc, overflow);
    if (rc) return rc;
    const size_t per = (size_t)(d->Cin / d->groups) * d->kD * d->kH * d->kW;
    for (int co = 0; co < d->Cout; ++co)
        for (size_t i = 0; i < per; ++i) dW[co * per + i] = dq2(acc[co * per + i], s_x, s_chan[co]);
    return REF_OK;
}
