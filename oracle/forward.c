/*
 * CPU oracle for the CNN forward pass -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain definitions, direct nested loops over NCHW tensors and OIHW weights,
 * accumulation in double, one rounding to float per output element (and, in
 * bf16 mode, a second rounding of that float to bfloat16, nearest-even).
 * Nothing here is tiled, fused or reordered, and nothing is shared with the HIP
 * library.  Only tests, the smoke check and the benchmark's cpu_baseline leg
 * may call this file.
 *
 * The paper (Sec. I, Sec. V) treats a DNN as an opaque sequence of vendor
 * kernels; what a layer computes is therefore the textbook definition:
 *   conv : Y[co,y,x] = b[co] + sum_{ci,ky,kx} W[co,ci,ky,kx] * Xpad[g*Cg+ci, y*s+ky-p, x*s+kx-p]
 *          (cross-correlation, zero padding, Hout = floor((H+2p-k)/s)+1)
 *   then  Y += R (optional residual), then ReLU / ReLU6.
 *   max-pool pads with -inf; global average = sum / (H*W); FC = mat-vec + bias.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* float -> bfloat16 (round to nearest, ties to even) -> float. NaN stays NaN. */
float orc_bf16_round_scalar(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) == 0x7f800000u && (u & 0x007fffffu)) { /* NaN: keep quiet NaN */
        u |= 0x00400000u;
        u &= 0xffff0000u;
    } else {
        uint32_t lsb = (u >> 16) & 1u;
        u += 0x7fffu + lsb;
        u &= 0xffff0000u;
    }
    memcpy(&f, &u, 4);
    return f;
}

void orc_bf16_round(float* x, int64_t n) {
    for (int64_t i = 0; i < n; ++i) x[i] = orc_bf16_round_scalar(x[i]);
}

static inline float finish(double acc, int act, int round_bf16) {
    if (act == 1) acc = acc > 0.0 ? acc : 0.0;
    else if (act == 2) acc = acc < 0.0 ? 0.0 : (acc > 6.0 ? 6.0 : acc);
    float f = (float)acc;
    return round_bf16 ? orc_bf16_round_scalar(f) : f;
}

/* x: [C][H][W]; w: [Cout][C/groups][k][k]; b: [Cout] or NULL; res: [Cout][Ho][Wo] or NULL; y: [Cout][Ho][Wo] */
void orc_conv2d(const float* x, int C, int H, int W, const float* w, const float* b, int Cout, int k,
                int stride, int pad, int groups, const float* res, int act, int round_bf16, float* y) {
    const int Ho = (H + 2 * pad - k) / stride + 1;
    const int Wo = (W + 2 * pad - k) / stride + 1;
    const int Cg = C / groups;       /* input channels per group  */
    const int Og = Cout / groups;    /* output channels per group */
#pragma omp parallel for schedule(dynamic, 1)
    for (int co = 0; co < Cout; ++co) {
        const int g = co / Og;
        for (int oy = 0; oy < Ho; ++oy) {
            for (int ox = 0; ox < Wo; ++ox) {
                double acc = b ? (double)b[co] : 0.0;
                for (int ci = 0; ci < Cg; ++ci) {
                    for (int ky = 0; ky < k; ++ky) {
                        const int iy = oy * stride + ky - pad;
                        if (iy < 0 || iy >= H) continue;           /* zero padding */
                        for (int kx = 0; kx < k; ++kx) {
                            const int ix = ox * stride + kx - pad;
                            if (ix < 0 || ix >= W) continue;
                            acc += (double)w[(((int64_t)co * Cg + ci) * k + ky) * k + kx] *
                                   (double)x[((int64_t)(g * Cg + ci) * H + iy) * W + ix];
                        }
                    }
                }
                const int64_t o = ((int64_t)co * Ho + oy) * Wo + ox;
                if (res) acc += (double)res[o];
                y[o] = finish(acc, act, round_bf16);
            }
        }
    }
}

void orc_maxpool2d(const float* x, int C, int H, int W, int k, int stride, int pad, float* y) {
    const int Ho = (H + 2 * pad - k) / stride + 1;
    const int Wo = (W + 2 * pad - k) / stride + 1;
    for (int c = 0; c < C; ++c)
        for (int oy = 0; oy < Ho; ++oy)
            for (int ox = 0; ox < Wo; ++ox) {
                float m = -INFINITY;
                for (int ky = 0; ky < k; ++ky) {
                    const int iy = oy * stride + ky - pad;
                    if (iy < 0 || iy >= H) continue;
                    for (int kx = 0; kx < k; ++kx) {
                        const int ix = ox * stride + kx - pad;
                        if (ix < 0 || ix >= W) continue;
                        const float v = x[((int64_t)c * H + iy) * W + ix];
                        if (v > m) m = v;
                    }
                }
                y[((int64_t)c * Ho + oy) * Wo + ox] = m;
            }
}

void orc_gavgpool(const float* x, int C, int H, int W, int round_bf16, float* y) {
    for (int c = 0; c < C; ++c) {
        double s = 0.0;
        for (int i = 0; i < H * W; ++i) s += (double)x[(int64_t)c * H * W + i];
        y[c] = finish(s / (double)(H * W), 0, round_bf16);
    }
}

/* y[o] = act(b[o] + sum_i w[o][i] x[i]) */
void orc_fc(const float* x, int K, const float* w, const float* b, int N, int act, int round_bf16, float* y) {
#pragma omp parallel for schedule(static)
    for (int o = 0; o < N; ++o) {
        double acc = b ? (double)b[o] : 0.0;
        for (int i = 0; i < K; ++i) acc += (double)w[(int64_t)o * K + i] * (double)x[i];
        y[o] = finish(acc, act, round_bf16);
    }
}

/* Unfused batch normalisation, used only to pin the weight-folding helper of the workload generator. */
void orc_batchnorm(const double* x, int C, int HW, const double* gamma, const double* beta, const double* mean,
                   const double* var, double eps, double* y) {
    for (int c = 0; c < C; ++c)
        for (int i = 0; i < HW; ++i)
            y[(int64_t)c * HW + i] = (x[(int64_t)c * HW + i] - mean[c]) / sqrt(var[c] + eps) * gamma[c] + beta[c];
}
