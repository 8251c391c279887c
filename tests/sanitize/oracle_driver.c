/* Runs every routine of the CPU oracle on small, ragged inputs.  Built with -fsanitize=address,undefined by
 * tests/test_sanitizers.py: an out-of-bounds index, a signed overflow or a misaligned access in the oracle's loops
 * aborts the run.  Results are not checked here (the pins do that); the checksum only keeps the calls alive. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "../../oracle/daq_ref.c"

static uint64_t lcg = 88172645463325252ull;
static float frand(void) {
    lcg = lcg * 6364136223846793005ull + 1442695040888963407ull;
    return (float)((double)(lcg >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}
static int8_t crand(void) { return (int8_t)(int)(frand() * 127.0f); }

int main(void) {
    double sum = 0.0;
    /* quantizer pieces */
    for (int i = 0; i < 2000; ++i) {
        float x = frand() * 3.0f, s = fabsf(frand()) + 1e-3f;
        sum += daq_ref_quantize_one(x, s, i & 1, daq_ref_uniform16((uint64_t)i * 77u, (uint32_t)(i & 1), (uint64_t)i));
        sum += daq_ref_dequantize_one((int8_t)(i % 255 - 127), s);
        sum += daq_ref_clip_value(i & 1, s, frand(), 1.0f + (float)(i % 3) * 0.25f, 0.8f);
        sum += daq_ref_classify((uint32_t)i, 2000.0, 0.3f);
    }
    {
        const int N = 3, C = 5, H = 7, W = 9, n = N * C * H * W;
        float* g = malloc(sizeof(float) * n);
        for (int i = 0; i < n; ++i) g[i] = frand() * 0.01f * (float)(1 + i % C);
        float gmax[5], mean[5], sigma[5], st[5] = {0, 1e-3f, -1.0f, 5.0f, 0}, s_chan[5], s_glob, stats[20];
        uint32_t cnt[5];
        uint8_t cls[5], frag[5];
        int8_t* vq = malloc(n);
        int8_t* qg = malloc(n);
        sum += daq_ref_channel_stats(g, N, C, H, W, gmax, mean, sigma) + daq_ref_tail_count(g, N, C, H, W, sigma, cnt);
        for (int scheme = 0; scheme < 4; ++scheme)
            for (int mode = 0; mode < 2; ++mode)
                sum += daq_ref_quantize_grad_scheme(g, N, C, H, W, st, 1.5f, 0.8f, 0.3f, mode, 42u + (uint64_t)scheme, scheme, vq, qg, s_chan,
                                                    &s_glob, cls, stats, frag);
        sum += daq_ref_quantize_grad(g, N, C, H, W, st, 1.0f, 0.8f, 0.3f, 0, 0u, vq, qg, s_chan, &s_glob, cls, stats, frag);
        float lg, lm, ls;
        sum += daq_ref_layer_stats(g, (size_t)n, &lg, &lm, &ls);
        double err[5 * 7];
        float bs[5];
        int32_t bj[5];
        sum += daq_ref_clip_search(g, N, C, H, W, 2.0f, 7, err, bs, bj) + bj[4];
        float sq;
        sum += daq_ref_quantize_tensor(g, (size_t)n, vq, &sq);
        free(g); free(vq); free(qg);
    }
    /* 2-D convolutions over strides, paddings, dilations and groups */
    const int cases[][10] = {{2, 3, 5, 6, 4, 3, 1, 1, 1, 1}, {1, 4, 7, 5, 6, 3, 2, 1, 1, 2}, {2, 2, 9, 9, 3, 7, 2, 3, 1, 1},
                             {1, 4, 6, 6, 4, 3, 1, 2, 2, 4}, {1, 2, 6, 5, 3, 3, 1, 3, 1, 1}, {2, 6, 4, 4, 9, 1, 2, 0, 1, 3}};
    for (unsigned c = 0; c < sizeof(cases) / sizeof(cases[0]); ++c) {
        const int* k = cases[c];
        ref_conv_desc d = {k[0], k[1], k[2], k[3], k[4], k[5], k[5], k[6], k[6], k[7], k[7], k[8], k[8], k[9]};
        const int Ho = daq_ref_out_h(&d), Wo = daq_ref_out_w(&d);
        const size_t nx = (size_t)d.N * d.Cin * d.Hin * d.Win, ny = (size_t)d.N * d.Cout * Ho * Wo,
                     nw = (size_t)d.Cout * (d.Cin / d.groups) * d.kH * d.kW;
        int8_t *qX = malloc(nx), *qG = malloc(ny), *qW = malloc(nw);
        float *X = malloc(4 * nx), *Wt = malloc(4 * nw), *Y = malloc(4 * ny), *dX = malloc(4 * nx), *dW = malloc(4 * nw), *sc = malloc(4 * d.Cout);
        int32_t *aY = malloc(4 * ny), *aX = malloc(4 * nx), *aW = malloc(4 * nw);
        for (size_t i = 0; i < nx; ++i) { qX[i] = crand(); X[i] = frand(); }
        for (size_t i = 0; i < ny; ++i) qG[i] = crand();
        for (size_t i = 0; i < nw; ++i) { qW[i] = crand(); Wt[i] = frand() * 0.1f; }
        for (int i = 0; i < d.Cout; ++i) sc[i] = fabsf(frand()) + 1e-4f;
        int ovf = 0;
        float sx, sw;
        sum += daq_ref_conv_fwd_acc(&d, qX, qW, aY, &ovf) + daq_ref_conv_bwd_data_acc(&d, qG, qW, aX, &ovf) +
               daq_ref_conv_bwd_filter_acc(&d, qX, qG, aW, &ovf);
        int64_t idx[3] = {0, (int64_t)nx - 1, (int64_t)nx / 2}, idw[3] = {0, (int64_t)nw - 1, (int64_t)nw / 2},
                idy[3] = {0, (int64_t)ny - 1, (int64_t)ny / 2};
        int32_t o3[3];
        sum += daq_ref_conv_bwd_data_acc_at(&d, qG, qW, idx, 3, o3) + daq_ref_conv_bwd_filter_acc_at(&d, qX, qG, idw, 3, o3) +
               daq_ref_conv_fwd_acc_at(&d, qX, qW, idy, 3, o3) + o3[1];
        int8_t *q2 = malloc(nx), *w2 = malloc(nw);
        sum += daq_ref_conv_fwd_int8(&d, X, Wt, q2, w2, &sx, &sw, Y, aY, &ovf) + daq_ref_conv_bwd_data_int8(&d, qG, 0.03f, qW, 0.1f, dX, aX, &ovf) +
               daq_ref_conv_bwd_filter_int8(&d, qX, 2.5f, qG, sc, dW, aW, &ovf) + daq_ref_dequantize_acc(aW, (int64_t)(nw < (size_t)d.Cout ? nw : (size_t)d.Cout), 2.5f, sc, dW);
        if (d.groups == d.Cin && d.groups == d.Cout) sum += daq_ref_conv_bwd_data_int8_chan(&d, qG, sc, qW, 0.1f, dX, aX, &ovf);
        sum += Y[ny - 1] + dX[nx - 1] + dW[nw - 1];
        free(qX); free(qG); free(qW); free(X); free(Wt); free(Y); free(dX); free(dW); free(sc); free(aY); free(aX); free(aW); free(q2); free(w2);
    }
    /* 3-D convolutions */
    const int c3[][19] = {{2, 3, 5, 6, 5, 4, 3, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1}, {1, 4, 7, 6, 6, 6, 3, 3, 3, 2, 2, 1, 1, 0, 2, 2, 1, 1, 2},
                          {1, 2, 3, 4, 5, 2, 3, 3, 3, 1, 1, 1, 3, 3, 3, 1, 1, 1, 1}};
    for (unsigned c = 0; c < sizeof(c3) / sizeof(c3[0]); ++c) {
        const int* k = c3[c];
        ref_conv3d_desc d = {k[0], k[1], k[2], k[3], k[4], k[5], k[6], k[7], k[8], k[9], k[10], k[11], k[12], k[13], k[14], k[15], k[16], k[17], k[18]};
        const size_t nx = (size_t)d.N * d.Cin * d.Din * d.Hin * d.Win,
                     ny = (size_t)d.N * d.Cout * daq_ref_out_d3(&d) * daq_ref_out_h3(&d) * daq_ref_out_w3(&d),
                     nw = (size_t)d.Cout * (d.Cin / d.groups) * d.kD * d.kH * d.kW;
        int8_t *qX = malloc(nx), *qG = malloc(ny), *qW = malloc(nw);
        float *X = malloc(4 * nx), *Wt = malloc(4 * nw), *Y = malloc(4 * ny), *dX = malloc(4 * nx), *dW = malloc(4 * nw), *sc = malloc(4 * d.Cout);
        int32_t *aY = malloc(4 * ny), *aX = malloc(4 * nx), *aW = malloc(4 * nw);
        for (size_t i = 0; i < nx; ++i) { qX[i] = crand(); X[i] = frand(); }
        for (size_t i = 0; i < ny; ++i) qG[i] = crand();
        for (size_t i = 0; i < nw; ++i) { qW[i] = crand(); Wt[i] = frand() * 0.1f; }
        for (int i = 0; i < d.Cout; ++i) sc[i] = fabsf(frand()) + 1e-4f;
        int ovf = 0;
        float sx, sw;
        int8_t *q2 = malloc(nx), *w2 = malloc(nw);
        sum += daq_ref_conv3d_fwd_int8(&d, X, Wt, q2, w2, &sx, &sw, Y, aY, &ovf) + daq_ref_conv3d_bwd_data_int8(&d, qG, 0.03f, qW, 0.1f, dX, aX, &ovf) +
               daq_ref_conv3d_bwd_filter_int8(&d, qX, 2.5f, qG, sc, dW, aW, &ovf);
        sum += Y[ny - 1] + dX[nx - 1] + dW[nw - 1];
        free(qX); free(qG); free(qW); free(X); free(Wt); free(Y); free(dX); free(dW); free(sc); free(aY); free(aX); free(aW); free(q2); free(w2);
    }
    printf("oracle sanitizer run ok (%g)\n", sum);
    return 0;
}
