/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain nested-loop definitions, in fp64, of every operation on the per-device
 * compute path of the 3D U-Net of LAMP (arXiv 2006.12575, Sec. 2.2 Eq. 2; channel
 * schedule in Sec. 3).  The paper fixes the network topology but not the layer
 * arithmetic; the layers are the textbook ones (3x3x3 cross-correlation with zero
 * padding 1, instance normalisation with biased variance, ReLU, 2x2x2 max pooling,
 * 2x2x2 stride-2 transposed convolution).  Every function below is the definition
 * written out once, with no blocking, no fusion and no reordering, so it can be
 * checked by eye.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may use this
 * file.  It shares no code with the HIP library and the product never calls it.
 *
 * Layout everywhere: activations are dense NDHWC (channel fastest), all double.
 *   conv weight            W [Co][3][3][3][Ci]
 *   transposed-conv weight Wt[Ci][2][2][2][Co]
 *
 * Parity pins (tests marked "not gpu"): brute-force scatter form, delta kernels,
 * all-ones closed form, 1x1x1 == matmul, adjoint and bilinear identities, finite
 * differences, normalisation invariants, routing invariants.  No function here is
 * "parity unpinned" with respect to the mathematics; the paper prints no numeric
 * value for any of them.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

typedef int64_t i64;

int ora_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static inline i64 vox(i64 n, i64 d, i64 h, i64 w, i64 D, i64 H, i64 W)
{
    return ((n * D + d) * H + h) * W + w;
}

/* O1: z[n,d,h,w,co] = b[co] + sum_{kd,kh,kw} sum_ci x[n,d+kd-1,h+kh-1,w+kw-1,ci] * W[co,kd,kh,kw,ci]
 * (cross-correlation, reads outside the volume are 0).  b may be NULL. */
void ora_conv3d_fwd(const double *x, const double *w, const double *b, double *z,
                    i64 N, i64 D, i64 H, i64 W, i64 Ci, i64 Co)
{
#pragma omp parallel for collapse(3) schedule(static)
    for (i64 n = 0; n < N; ++n)
        for (i64 d = 0; d < D; ++d)
            for (i64 h = 0; h < H; ++h)
                for (i64 wv = 0; wv < W; ++wv)
                    for (i64 co = 0; co < Co; ++co) {
                        double acc = b ? b[co] : 0.0;
                        for (i64 kd = 0; kd < 3; ++kd)
                            for (i64 kh = 0; kh < 3; ++kh)
                                for (i64 kw = 0; kw < 3; ++kw) {
                                    i64 id = d + kd - 1, ih = h + kh - 1, iw = wv + kw - 1;
                                    if (id < 0 || id >= D || ih < 0 || ih >= H || iw < 0 || iw >= W)
                                        continue;
                                    const double *xp = x + vox(n, id, ih, iw, D, H, W) * Ci;
                                    const double *wp = w + (((co * 3 + kd) * 3 + kh) * 3 + kw) * Ci;
                                    for (i64 ci = 0; ci < Ci; ++ci)
                                        acc += xp[ci] * wp[ci];
                                }
                        z[vox(n, d, h, wv, D, H, W) * Co + co] = acc;
                    }
}

/* O2: dx[n,i,j,k,ci] = sum_{kd,kh,kw} sum_co dz[n,i-kd+1,j-kh+1,k-kw+1,co] * W[co,kd,kh,kw,ci]
 * (the adjoint of O1 with respect to x; the paper's B_k of Sec. 2.1). */
void ora_conv3d_dgrad(const double *dz, const double *w, double *dx,
                      i64 N, i64 D, i64 H, i64 W, i64 Ci, i64 Co)
{
#pragma omp parallel for collapse(3) schedule(static)
    for (i64 n = 0; n < N; ++n)
        for (i64 i = 0; i < D; ++i)
            for (i64 j = 0; j < H; ++j)
                for (i64 k = 0; k < W; ++k)
                    for (i64 ci = 0; ci < Ci; ++ci) {
                        double acc = 0.0;
                        for (i64 kd = 0; kd < 3; ++kd)
                            for (i64 kh = 0; kh < 3; ++kh)
                                for (i64 kw = 0; kw < 3; ++kw) {
                                    i64 od = i - kd + 1, oh = j - kh + 1, ow = k - kw + 1;
                                    if (od < 0 || od >= D || oh < 0 || oh >= H || ow < 0 || ow >= W)
                                        continue;
                                    const double *gp = dz + vox(n, od, oh, ow, D, H, W) * Co;
                                    for (i64 co = 0; co < Co; ++co)
                                        acc += gp[co] * w[(((co * 3 + kd) * 3 + kh) * 3 + kw) * Ci + ci];
                                }
                        dx[vox(n, i, j, k, D, H, W) * Ci + ci] = acc;
                    }
}

/* O3: dW[co,kd,kh,kw,ci] = beta*dW + sum_n sum_{d,h,w} dz[n,d,h,w,co] * x[n,d+kd-1,h+kh-1,w+kw-1,ci]
 *     db[co] = beta*db + sum dz[...,co]      (db may be NULL)
 * beta = 1 is the synchronous accumulation over micro-batches of Sec. 2.1. */
void ora_conv3d_wgrad(const double *x, const double *dz, double *dw, double *db, double beta,
                      i64 N, i64 D, i64 H, i64 W, i64 Ci, i64 Co)
{
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (i64 co = 0; co < Co; ++co)
        for (i64 t = 0; t < 27; ++t) {
            i64 kd = t / 9, kh = (t / 3) % 3, kw = t % 3;
            for (i64 ci = 0; ci < Ci; ++ci) {
                double acc = 0.0;
                for (i64 n = 0; n < N; ++n)
                    for (i64 d = 0; d < D; ++d)
                        for (i64 h = 0; h < H; ++h)
                            for (i64 wv = 0; wv < W; ++wv) {
                                i64 id = d + kd - 1, ih = h + kh - 1, iw = wv + kw - 1;
                                if (id < 0 || id >= D || ih < 0 || ih >= H || iw < 0 || iw >= W)
                                    continue;
                                acc += dz[vox(n, d, h, wv, D, H, W) * Co + co] *
                                       x[vox(n, id, ih, iw, D, H, W) * Ci + ci];
                            }
                i64 o = (co * 27 + t) * Ci + ci;
                dw[o] = (beta != 0.0 ? beta * dw[o] : 0.0) + acc;
            }
        }
    if (db) {
        for (i64 co = 0; co < Co; ++co) {
            double acc = 0.0;
            for (i64 v = 0; v < N * D * H * W; ++v)
                acc += dz[v * Co + co];
            db[co] = (beta != 0.0 ? beta * db[co] : 0.0) + acc;
        }
    }
}

/* O4: per (n,c) over the V = D*H*W voxels:
 *   mu = sum z / V ; var = sum (z-mu)^2 / V (biased) ; rstd = 1/sqrt(var+eps)
 *   y = max(0, gamma_c * (z-mu)*rstd + beta_c)
 * gamma/beta NULL mean 1/0.  stats (nullable) receives [N][C][2] = (mu, rstd).
 * relu = 0 skips the max (normalisation only). */
void ora_inorm_relu(const double *z, const double *gamma, const double *beta, double eps,
                    double *y, double *stats, i64 N, i64 V, i64 C, int relu)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (i64 n = 0; n < N; ++n)
        for (i64 c = 0; c < C; ++c) {
            const double *zp = z + n * V * C + c;
            double s = 0.0;
            for (i64 v = 0; v < V; ++v)
                s += zp[v * C];
            double mu = s / (double)V;
            double q = 0.0;
            for (i64 v = 0; v < V; ++v) {
                double t = zp[v * C] - mu;
                q += t * t;
            }
            double rstd = 1.0 / sqrt(q / (double)V + eps);
            double g = gamma ? gamma[c] : 1.0, bt = beta ? beta[c] : 0.0;
            double *yp = y + n * V * C + c;
            for (i64 v = 0; v < V; ++v) {
                double u = g * ((zp[v * C] - mu) * rstd) + bt;
                yp[v * C] = (relu && !(u > 0.0)) ? 0.0 : u;
            }
            if (stats) {
                stats[(n * C + c) * 2 + 0] = mu;
                stats[(n * C + c) * 2 + 1] = rstd;
            }
        }
}

/* O5: backward of O4.  With zh = (z-mu)*rstd, u = gamma*zh + beta, g = dy*[u>0]:
 *   dbeta_c  (+)= sum_{n,v} g ;  dgamma_c (+)= sum_{n,v} g*zh
 *   dz = gamma*rstd*( g - mean_v(g) - zh*mean_v(g*zh) )       per (n,c)
 * dgamma/dbeta nullable; when given they are overwritten (summed over n). */
void ora_inorm_relu_bwd(const double *dy, const double *z, const double *gamma, const double *beta,
                        double eps, double *dz, double *dgamma, double *dbeta,
                        i64 N, i64 V, i64 C, int relu)
{
    if (dgamma) memset(dgamma, 0, sizeof(double) * (size_t)C);
    if (dbeta) memset(dbeta, 0, sizeof(double) * (size_t)C);
#pragma omp parallel for schedule(static)
    for (i64 c = 0; c < C; ++c)
        for (i64 n = 0; n < N; ++n) {
            const double *zp = z + n * V * C + c;
            const double *gp = dy + n * V * C + c;
            double s = 0.0;
            for (i64 v = 0; v < V; ++v)
                s += zp[v * C];
            double mu = s / (double)V;
            double q = 0.0;
            for (i64 v = 0; v < V; ++v) {
                double t = zp[v * C] - mu;
                q += t * t;
            }
            double rstd = 1.0 / sqrt(q / (double)V + eps);
            double g = gamma ? gamma[c] : 1.0, bt = beta ? beta[c] : 0.0;
            double sg = 0.0, sgz = 0.0;
            for (i64 v = 0; v < V; ++v) {
                double zh = (zp[v * C] - mu) * rstd;
                double u = g * zh + bt;
                double gg = (relu && !(u > 0.0)) ? 0.0 : gp[v * C];
                sg += gg;
                sgz += gg * zh;
            }
            double mg = sg / (double)V, mgz = sgz / (double)V;
            double *op = dz + n * V * C + c;
            for (i64 v = 0; v < V; ++v) {
                double zh = (zp[v * C] - mu) * rstd;
                double u = g * zh + bt;
                double gg = (relu && !(u > 0.0)) ? 0.0 : gp[v * C];
                op[v * C] = g * rstd * (gg - mg - zh * mgz);
            }
            if (dbeta) dbeta[c] += sg;
            if (dgamma) dgamma[c] += sgz;
        }
}

/* O6: y[n,d,h,w,c] = max_{i,j,k in {0,1}} x[n,2d+i,2h+j,2w+k,c]   (D,H,W even). */
void ora_maxpool2_fwd(const double *x, double *y, i64 N, i64 D, i64 H, i64 W, i64 C)
{
    i64 Do = D / 2, Ho = H / 2, Wo = W / 2;
#pragma omp parallel for collapse(3) schedule(static)
    for (i64 n = 0; n < N; ++n)
        for (i64 d = 0; d < Do; ++d)
            for (i64 h = 0; h < Ho; ++h)
                for (i64 wv = 0; wv < Wo; ++wv)
                    for (i64 c = 0; c < C; ++c) {
                        double m = -INFINITY;
                        for (i64 i = 0; i < 2; ++i)
                            for (i64 j = 0; j < 2; ++j)
                                for (i64 k = 0; k < 2; ++k) {
                                    double v = x[vox(n, 2 * d + i, 2 * h + j, 2 * wv + k, D, H, W) * C + c];
                                    if (v > m) m = v;
                                }
                        y[vox(n, d, h, wv, Do, Ho, Wo) * C + c] = m;
                    }
}

/* O6 backward: dy goes to the arg-max of the window, the first one in (i,j,k)
 * raster order under strict '>' ; every other position of the window gets 0. */
void ora_maxpool2_bwd(const double *x, const double *dy, double *dx, i64 N, i64 D, i64 H, i64 W, i64 C)
{
    i64 Do = D / 2, Ho = H / 2, Wo = W / 2;
    memset(dx, 0, sizeof(double) * (size_t)(N * D * H * W * C));
#pragma omp parallel for collapse(3) schedule(static)
    for (i64 n = 0; n < N; ++n)
        for (i64 d = 0; d < Do; ++d)
            for (i64 h = 0; h < Ho; ++h)
                for (i64 wv = 0; wv < Wo; ++wv)
                    for (i64 c = 0; c < C; ++c) {
                        double m = -INFINITY;
                        i64 arg = -1;
                        for (i64 i = 0; i < 2; ++i)
                            for (i64 j = 0; j < 2; ++j)
                                for (i64 k = 0; k < 2; ++k) {
                                    i64 a = vox(n, 2 * d + i, 2 * h + j, 2 * wv + k, D, H, W) * C + c;
                                    if (x[a] > m) {
                                        m = x[a];
                                        arg = a;
                                    }
                                }
                        if (arg >= 0) dx[arg] = dy[vox(n, d, h, wv, Do, Ho, Wo) * C + c];
                    }
}

/* O7: y[n,2d+i,2h+j,2w+k,co] = b[co] + sum_ci x[n,d,h,w,ci] * Wt[ci,i,j,k,co]
 * x is [N,D,H,W,Ci]; y is [N,2D,2H,2W,Co]; b may be NULL. */
void ora_convtr3d_fwd(const double *x, const double *wt, const double *b, double *y,
                      i64 N, i64 D, i64 H, i64 W, i64 Ci, i64 Co)
{
#pragma omp parallel for collapse(3) schedule(static)
    for (i64 n = 0; n < N; ++n)
        for (i64 d = 0; d < D; ++d)
            for (i64 h = 0; h < H; ++h)
                for (i64 wv = 0; wv < W; ++wv)
                    for (i64 i = 0; i < 2; ++i)
                        for (i64 j = 0; j < 2; ++j)
                            for (i64 k = 0; k < 2; ++k)
                                for (i64 co = 0; co < Co; ++co) {
                                    double acc = b ? b[co] : 0.0;
                                    const double *xp = x + vox(n, d, h, wv, D, H, W) * Ci;
                                    for (i64 ci = 0; ci < Ci; ++ci)
                                        acc += xp[ci] * wt[(((ci * 2 + i) * 2 + j) * 2 + k) * Co + co];
                                    y[vox(n, 2 * d + i, 2 * h + j, 2 * wv + k, 2 * D, 2 * H, 2 * W) * Co + co] = acc;
                                }
}

/* O7 backward:
 *   dx[n,d,h,w,ci]    = sum_{i,j,k,co} dy[n,2d+i,2h+j,2w+k,co] * Wt[ci,i,j,k,co]
 *   dWt[ci,i,j,k,co]  = beta*dWt + sum_{n,d,h,w} x[n,d,h,w,ci] * dy[n,2d+i,2h+j,2w+k,co]
 *   db[co]            = beta*db  + sum dy[...,co]
 * Each of dx, dwt, db may be NULL (skipped). */
void ora_convtr3d_bwd(const double *x, const double *wt, const double *dy,
                      double *dx, double *dwt, double *db, double beta,
                      i64 N, i64 D, i64 H, i64 W, i64 Ci, i64 Co)
{
    if (dx) {
#pragma omp parallel for collapse(3) schedule(static)
        for (i64 n = 0; n < N; ++n)
            for (i64 d = 0; d < D; ++d)
                for (i64 h = 0; h < H; ++h)
                    for (i64 wv = 0; wv < W; ++wv)
                        for (i64 ci = 0; ci < Ci; ++ci) {
                            double acc = 0.0;
                            for (i64 i = 0; i < 2; ++i)
                                for (i64 j = 0; j < 2; ++j)
                                    for (i64 k = 0; k < 2; ++k) {
                                        const double *gp =
                                            dy + vox(n, 2 * d + i, 2 * h + j, 2 * wv + k, 2 * D, 2 * H, 2 * W) * Co;
                                        const double *wp = wt + (((ci * 2 + i) * 2 + j) * 2 + k) * Co;
                                        for (i64 co = 0; co < Co; ++co)
                                            acc += gp[co] * wp[co];
                                    }
                            dx[vox(n, d, h, wv, D, H, W) * Ci + ci] = acc;
                        }
    }
    if (dwt) {
#pragma omp parallel for collapse(2) schedule(static)
        for (i64 ci = 0; ci < Ci; ++ci)
            for (i64 t = 0; t < 8; ++t) {
                i64 i = t / 4, j = (t / 2) % 2, k = t % 2;
                for (i64 co = 0; co < Co; ++co) {
                    double acc = 0.0;
                    for (i64 n = 0; n < N; ++n)
                        for (i64 d = 0; d < D; ++d)
                            for (i64 h = 0; h < H; ++h)
                                for (i64 wv = 0; wv < W; ++wv)
                                    acc += x[vox(n, d, h, wv, D, H, W) * Ci + ci] *
                                           dy[vox(n, 2 * d + i, 2 * h + j, 2 * wv + k, 2 * D, 2 * H, 2 * W) * Co + co];
                    i64 o = (ci * 8 + t) * Co + co;
                    dwt[o] = (beta != 0.0 ? beta * dwt[o] : 0.0) + acc;
                }
            }
    }
    if (db) {
        for (i64 co = 0; co < Co; ++co) {
            double acc = 0.0;
            for (i64 v = 0; v < N * 8 * D * H * W; ++v)
                acc += dy[v * Co + co];
            db[co] = (beta != 0.0 ? beta * db[co] : 0.0) + acc;
        }
    }
}
