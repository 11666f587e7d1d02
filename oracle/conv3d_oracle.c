/*
 * fp64 CPU oracle for the 3-D convolution and its two gradients.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may call into this
 * file; it exists so that the GPU kernels can be compared with a plain,
 * slow, obviously correct statement of what they must compute.  It shares no
 * code, header, table or helper with the HIP library.
 *
 * What is computed.  The paper trains a 3D U-Net whose layers produce a
 * feature map A^l in the forward pass that the same layer needs again in the
 * backward pass (Section 3.1, Fig. 1); it delegates the convolutions to a
 * closed vendor library (Section 4.1) and states no formula for them.  The
 * operation is therefore the textbook one, written out as nested loops:
 *
 *   activations  NDHWC                      x[n][d][h][w][ci]
 *   weights      [Cout][kD][kH][kW][Cin]    w[co][kd][kh][kw][ci]
 *   zero padding p per side, stride s, cross-correlation (no kernel flip)
 *   Do = floor((D + 2 pD - kD) / sD) + 1, likewise Ho, Wo
 *
 *   forward   y[n,o,co]  = sum_{t,ci} x[n, o*s - p + t, ci] * w[co,t,ci]
 *   data-grad dx[n,i,ci] = sum over (o,t,co) with o*s - p + t == i of
 *                          dy[n,o,co] * w[co,t,ci]      (adjoint in x)
 *   wt-grad   dw[co,t,ci]= sum_{n,o} dy[n,o,co] * x[n, o*s - p + t, ci]
 *
 * x outside [0,D)x[0,H)x[0,W) counts as zero.  All sums run in double, in
 * the loop order written; there is no blocking or fusion.
 *
 * The *_at functions evaluate single output elements of the same three
 * definitions (inputs given as float holding exactly-representable values,
 * widened to double before any arithmetic) so that full-size volumes can be
 * spot-checked in seconds.  dgrad is a scatter in the full function and a
 * gather in dgrad_at, on purpose: tests require the two to agree.
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>

typedef struct {
    int N, D, H, W, Cin;
    int Cout, kD, kH, kW;
    int sD, sH, sW, pD, pH, pW;
} oracle_conv_shape;

static int out_extent(int in, int pad, int k, int s) { return (in + 2 * pad - k) / s + 1; }

int oracle_conv3d_out_dims(const oracle_conv_shape *g, int *Do, int *Ho, int *Wo)
{
    if (!g || g->N <= 0 || g->D <= 0 || g->H <= 0 || g->W <= 0 || g->Cin <= 0 || g->Cout <= 0) return -1;
    if (g->kD <= 0 || g->kH <= 0 || g->kW <= 0 || g->sD <= 0 || g->sH <= 0 || g->sW <= 0) return -1;
    if (g->pD < 0 || g->pH < 0 || g->pW < 0) return -1;
    if (g->D + 2 * g->pD < g->kD || g->H + 2 * g->pH < g->kH || g->W + 2 * g->pW < g->kW) return -1;
    *Do = out_extent(g->D, g->pD, g->kD, g->sD);
    *Ho = out_extent(g->H, g->pH, g->kH, g->sH);
    *Wo = out_extent(g->W, g->pW, g->kW, g->sW);
    return 0;
}

#define XIDX(g, n, d, h, w) (((((size_t)(n) * (g)->D + (d)) * (g)->H + (h)) * (g)->W + (w)) * (size_t)(g)->Cin)
#define YIDX(g, n, d, h, w, Do, Ho, Wo) (((((size_t)(n) * (Do) + (d)) * (Ho) + (h)) * (Wo) + (w)) * (size_t)(g)->Cout)
#define WIDX(g, co, kd, kh, kw) (((((size_t)(co) * (g)->kD + (kd)) * (g)->kH + (kh)) * (g)->kW + (kw)) * (size_t)(g)->Cin)

/* forward: one output element at a time, taps then input channels innermost */
int oracle_conv3d_fwd(const oracle_conv_shape *g, const double *x, const double *w, double *y)
{
    int Do, Ho, Wo;
    if (oracle_conv3d_out_dims(g, &Do, &Ho, &Wo)) return -1;
    long rows = (long)g->N * Do;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r) {
        int n = (int)(r / Do), od = (int)(r % Do);
        for (int oh = 0; oh < Ho; ++oh)
        for (int ow = 0; ow < Wo; ++ow)
        for (int co = 0; co < g->Cout; ++co) {
            double acc = 0.0;
            for (int kd = 0; kd < g->kD; ++kd) {
                int id = od * g->sD - g->pD + kd;
                if (id < 0 || id >= g->D) continue;
                for (int kh = 0; kh < g->kH; ++kh) {
                    int ih = oh * g->sH - g->pH + kh;
                    if (ih < 0 || ih >= g->H) continue;
                    for (int kw = 0; kw < g->kW; ++kw) {
                        int iw = ow * g->sW - g->pW + kw;
                        if (iw < 0 || iw >= g->W) continue;
                        const double *xp = x + XIDX(g, n, id, ih, iw);
                        const double *wp = w + WIDX(g, co, kd, kh, kw);
                        for (int ci = 0; ci < g->Cin; ++ci) acc += xp[ci] * wp[ci];
                    }
                }
            }
            y[YIDX(g, n, od, oh, ow, Do, Ho, Wo) + co] = acc;
        }
    }
    return 0;
}

/* data gradient as a scatter: every (output position, tap) pushes its
 * contribution into the input position it read in the forward pass.
 * Threads own disjoint input channels, so no two threads touch one dx. */
int oracle_conv3d_dgrad(const oracle_conv_shape *g, const double *dy, const double *w, double *dx)
{
    int Do, Ho, Wo;
    if (oracle_conv3d_out_dims(g, &Do, &Ho, &Wo)) return -1;
    memset(dx, 0, sizeof(double) * (size_t)g->N * g->D * g->H * g->W * g->Cin);
#pragma omp parallel for schedule(static)
    for (int ci = 0; ci < g->Cin; ++ci) {
        for (int n = 0; n < g->N; ++n)
        for (int od = 0; od < Do; ++od)
        for (int oh = 0; oh < Ho; ++oh)
        for (int ow = 0; ow < Wo; ++ow) {
            const double *gp = dy + YIDX(g, n, od, oh, ow, Do, Ho, Wo);
            for (int kd = 0; kd < g->kD; ++kd) {
                int id = od * g->sD - g->pD + kd;
                if (id < 0 || id >= g->D) continue;
                for (int kh = 0; kh < g->kH; ++kh) {
                    int ih = oh * g->sH - g->pH + kh;
                    if (ih < 0 || ih >= g->H) continue;
                    for (int kw = 0; kw < g->kW; ++kw) {
                        int iw = ow * g->sW - g->pW + kw;
                        if (iw < 0 || iw >= g->W) continue;
                        double acc = 0.0;
                        for (int co = 0; co < g->Cout; ++co)
                            acc += gp[co] * w[WIDX(g, co, kd, kh, kw) + ci];
                        dx[XIDX(g, n, id, ih, iw) + ci] += acc;
                    }
                }
            }
        }
    }
    return 0;
}

/* weight gradient: one dw element at a time, summed over batch and volume */
int oracle_conv3d_wgrad(const oracle_conv_shape *g, const double *x, const double *dy, double *dw)
{
    int Do, Ho, Wo;
    if (oracle_conv3d_out_dims(g, &Do, &Ho, &Wo)) return -1;
    long taps = (long)g->kD * g->kH * g->kW;
    long rows = (long)g->Cout * taps;
#pragma omp parallel for schedule(dynamic, 1)
    for (long r = 0; r < rows; ++r) {
        int co = (int)(r / taps);
        int t = (int)(r % taps);
        int kd = t / (g->kH * g->kW), kh = (t / g->kW) % g->kH, kw = t % g->kW;
        for (int ci = 0; ci < g->Cin; ++ci) {
            double acc = 0.0;
            for (int n = 0; n < g->N; ++n)
            for (int od = 0; od < Do; ++od) {
                int id = od * g->sD - g->pD + kd;
                if (id < 0 || id >= g->D) continue;
                for (int oh = 0; oh < Ho; ++oh) {
                    int ih = oh * g->sH - g->pH + kh;
                    if (ih < 0 || ih >= g->H) continue;
                    for (int ow = 0; ow < Wo; ++ow) {
                        int iw = ow * g->sW - g->pW + kw;
                        if (iw < 0 || iw >= g->W) continue;
                        acc += dy[YIDX(g, n, od, oh, ow, Do, Ho, Wo) + co] * x[XIDX(g, n, id, ih, iw) + ci];
                    }
                }
            }
            dw[WIDX(g, co, kd, kh, kw) + ci] = acc;
        }
    }
    return 0;
}

/* ---- single-element evaluations for spot checks on full-size volumes ---- */

/* y at flat NDHWC output indices idx[0..count) */
int oracle_conv3d_fwd_at(const oracle_conv_shape *g, const float *x, const float *w,
                         const int64_t *idx, long count, double *out)
{
    int Do, Ho, Wo;
    if (oracle_conv3d_out_dims(g, &Do, &Ho, &Wo)) return -1;
#pragma omp parallel for schedule(static)
    for (long q = 0; q < count; ++q) {
        int64_t r = idx[q];
        int co = (int)(r % g->Cout); r /= g->Cout;
        int ow = (int)(r % Wo); r /= Wo;
        int oh = (int)(r % Ho); r /= Ho;
        int od = (int)(r % Do); r /= Do;
        int n = (int)r;
        double acc = 0.0;
        for (int kd = 0; kd < g->kD; ++kd)
        for (int kh = 0; kh < g->kH; ++kh)
        for (int kw = 0; kw < g->kW; ++kw) {
            int id = od * g->sD - g->pD + kd, ih = oh * g->sH - g->pH + kh, iw = ow * g->sW - g->pW + kw;
            if (id < 0 || id >= g->D || ih < 0 || ih >= g->H || iw < 0 || iw >= g->W) continue;
            const float *xp = x + XIDX(g, n, id, ih, iw);
            const float *wp = w + WIDX(g, co, kd, kh, kw);
            for (int ci = 0; ci < g->Cin; ++ci) acc += (double)xp[ci] * (double)wp[ci];
        }
        out[q] = acc;
    }
    return 0;
}

/* dx at flat NDHWC input indices: gather over the (tap, output) pairs whose
 * forward read touched that input position */
int oracle_conv3d_dgrad_at(const oracle_conv_shape *g, const float *dy, const float *w,
                           const int64_t *idx, long count, double *out)
{
    int Do, Ho, Wo;
    if (oracle_conv3d_out_dims(g, &Do, &Ho, &Wo)) return -1;
#pragma omp parallel for schedule(static)
    for (long q = 0; q < count; ++q) {
        int64_t r = idx[q];
        int ci = (int)(r % g->Cin); r /= g->Cin;
        int iw = (int)(r % g->W); r /= g->W;
        int ih = (int)(r % g->H); r /= g->H;
        int id = (int)(r % g->D); r /= g->D;
        int n = (int)r;
        double acc = 0.0;
        for (int kd = 0; kd < g->kD; ++kd) {
            int nd = id + g->pD - kd;
            if (nd < 0 || nd % g->sD) continue;
            int od = nd / g->sD;
            if (od >= Do) continue;
            for (int kh = 0; kh < g->kH; ++kh) {
                int nh = ih + g->pH - kh;
                if (nh < 0 || nh % g->sH) continue;
                int oh = nh / g->sH;
                if (oh >= Ho) continue;
                for (int kw = 0; kw < g->kW; ++kw) {
                    int nw = iw + g->pW - kw;
                    if (nw < 0 || nw % g->sW) continue;
                    int ow = nw / g->sW;
                    if (ow >= Wo) continue;
                    const float *gp = dy + YIDX(g, n, od, oh, ow, Do, Ho, Wo);
                    for (int co = 0; co < g->Cout; ++co)
                        acc += (double)gp[co] * (double)w[WIDX(g, co, kd, kh, kw) + ci];
                }
            }
        }
        out[q] = acc;
    }
    return 0;
}

/* dw at flat [Cout][kD][kH][kW][Cin] indices; each is a full spatial sum */
int oracle_conv3d_wgrad_at(const oracle_conv_shape *g, const float *x, const float *dy,
                           const int64_t *idx, long count, double *out)
{
    int Do, Ho, Wo;
    if (oracle_conv3d_out_dims(g, &Do, &Ho, &Wo)) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (long q = 0; q < count; ++q) {
        int64_t r = idx[q];
        int ci = (int)(r % g->Cin); r /= g->Cin;
        int kw = (int)(r % g->kW); r /= g->kW;
        int kh = (int)(r % g->kH); r /= g->kH;
        int kd = (int)(r % g->kD); r /= g->kD;
        int co = (int)r;
        double acc = 0.0;
        for (int n = 0; n < g->N; ++n)
        for (int od = 0; od < Do; ++od) {
            int id = od * g->sD - g->pD + kd;
            if (id < 0 || id >= g->D) continue;
            for (int oh = 0; oh < Ho; ++oh) {
                int ih = oh * g->sH - g->pH + kh;
                if (ih < 0 || ih >= g->H) continue;
                for (int ow = 0; ow < Wo; ++ow) {
                    int iw = ow * g->sW - g->pW + kw;
                    if (iw < 0 || iw >= g->W) continue;
                    acc += (double)dy[YIDX(g, n, od, oh, ow, Do, Ho, Wo) + co] * (double)x[XIDX(g, n, id, ih, iw) + ci];
                }
            }
        }
        out[q] = acc;
    }
    return 0;
}

/* Decoder upsampling: 2x2x2-style transposed convolution with stride equal
 * to the kernel size and no padding, written directly (not via dgrad):
 *   u[n, j*k + t, co] = sum_ci z[n, j, ci] * v[ci][t][co]
 * z is [N][Dz][Hz][Wz][Ci], v is [Ci][kD][kH][kW][Co], u is
 * [N][Dz*kD][Hz*kH][Wz*kW][Co].  Every output voxel receives exactly one tap. */
int oracle_tconv3d_fwd(int N, int Dz, int Hz, int Wz, int Ci, int Co, int kD, int kH, int kW,
                       const double *z, const double *v, double *u)
{
    if (N <= 0 || Dz <= 0 || Hz <= 0 || Wz <= 0 || Ci <= 0 || Co <= 0 || kD <= 0 || kH <= 0 || kW <= 0) return -1;
    int Du = Dz * kD, Hu = Hz * kH, Wu = Wz * kW;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < (long)N * Du; ++r) {
        int n = (int)(r / Du), ud = (int)(r % Du);
        for (int uh = 0; uh < Hu; ++uh)
        for (int uw = 0; uw < Wu; ++uw) {
            int jd = ud / kD, td = ud % kD, jh = uh / kH, th = uh % kH, jw = uw / kW, tw = uw % kW;
            const double *zp = z + ((((size_t)n * Dz + jd) * Hz + jh) * Wz + jw) * (size_t)Ci;
            for (int co = 0; co < Co; ++co) {
                double acc = 0.0;
                for (int ci = 0; ci < Ci; ++ci)
                    acc += zp[ci] * v[((((size_t)ci * kD + td) * kH + th) * kW + tw) * (size_t)Co + co];
                u[((((size_t)n * Du + ud) * Hu + uh) * Wu + uw) * (size_t)Co + co] = acc;
            }
        }
    }
    return 0;
}
