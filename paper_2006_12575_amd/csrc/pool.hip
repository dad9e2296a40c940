// 2x2x2 max pooling (stride 2), forward and backward.  Bandwidth-bound; one thread per
// (output voxel, channel vector).
#include <initializer_list>
#include "internal.h"
#include "vec.h"

namespace lamp {

template <typename T, int VEC>
__global__ __launch_bounds__(256) void maxpool2_fwd_kernel(const T* __restrict__ x, int ldx, NormIn nm, T* __restrict__ y,
                                                           int ldy, int N, int Do, int Ho, int Wo, int C,
                                                           T* __restrict__ yfull = nullptr, int ldyf = 0) {
    const int CV = C / VEC;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = (int64_t)N * Do * Ho * Wo * CV;
    if (idx >= total) return;
    const int cv = (int)(idx % CV);
    int64_t ov = idx / CV;
    const int w = (int)(ov % Wo);
    int64_t r = ov / Wo;
    const int h = (int)(r % Ho);
    r /= Ho;
    const int d = (int)(r % Do);
    const int n = (int)(r / Do);
    const int H = 2 * Ho, W = 2 * Wo, D = 2 * Do;
    float m[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) m[i] = -INFINITY;
    if (yfull) {
        // also write the activated input: all channels normalised, the coefficients of this thread's channels
        // fetched once, the two voxels of a w pair stored back to back
        float a[VEC], b[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) norm_coeffs(nm, n, cv * VEC + e, a[e], b[e]);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int i = t >> 1, j = t & 1;
            const int64_t iv = (((int64_t)n * D + 2 * d + i) * H + 2 * h + j) * W + 2 * w;
            float v0[VEC], v1[VEC];
            Vec<T, VEC>::load(x + iv * ldx + cv * VEC, v0);
            Vec<T, VEC>::load(x + (iv + 1) * ldx + cv * VEC, v1);
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                float u0 = norm_u(v0[e], a[e], b[e]), u1 = norm_u(v1[e], a[e], b[e]);
                if (nm.relu) { u0 = u0 > 0.f ? u0 : 0.f; u1 = u1 > 0.f ? u1 : 0.f; }
                v0[e] = io<T>::rnd(u0); v1[e] = io<T>::rnd(u1);
                const float mm = v0[e] > v1[e] ? v0[e] : v1[e];
                m[e] = mm > m[e] ? mm : m[e];
            }
            Vec<T, VEC>::store(yfull + iv * ldyf + cv * VEC, v0);
            Vec<T, VEC>::store(yfull + (iv + 1) * ldyf + cv * VEC, v1);
        }
        Vec<T, VEC>::store(y + ov * ldy + cv * VEC, m);
        return;
    }
    for (int t = 0; t < 8; ++t) {
        int i = t >> 2, j = (t >> 1) & 1, k = t & 1;
        const T* p = x + ((((int64_t)n * D + 2 * d + i) * H + 2 * h + j) * W + 2 * w + k) * ldx + cv * VEC;
        float v[VEC];
        load_norm_vec<T, VEC>(p, nm, n, cv * VEC, v);
#pragma unroll
        for (int e = 0; e < VEC; ++e) m[e] = v[e] > m[e] ? v[e] : m[e];
    }
    Vec<T, VEC>::store(y + ov * ldy + cv * VEC, m);
}

template <typename T, int VEC>
__global__ __launch_bounds__(256) void maxpool2_bwd_kernel(const T* __restrict__ x, int ldx, NormIn nm,
                                                           const T* __restrict__ dy, int ldg, const T* __restrict__ add,
                                                           int lda, T* __restrict__ dx, int ldo, int N, int Do, int Ho,
                                                           int Wo, int C) {
    const int CV = C / VEC;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = (int64_t)N * Do * Ho * Wo * CV;
    if (idx >= total) return;
    const int cv = (int)(idx % CV);
    int64_t ov = idx / CV;
    const int w = (int)(ov % Wo);
    int64_t r = ov / Wo;
    const int h = (int)(r % Ho);
    r /= Ho;
    const int d = (int)(r % Do);
    const int n = (int)(r / Do);
    const int H = 2 * Ho, W = 2 * Wo, D = 2 * Do;
    float m[VEC];
    int arg[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) { m[i] = -INFINITY; arg[i] = 0; }
    for (int t = 0; t < 8; ++t) {
        int i = t >> 2, j = (t >> 1) & 1, k = t & 1;
        const T* p = x + ((((int64_t)n * D + 2 * d + i) * H + 2 * h + j) * W + 2 * w + k) * ldx + cv * VEC;
        float v[VEC];
        load_norm_vec<T, VEC>(p, nm, n, cv * VEC, v);
#pragma unroll
        for (int e = 0; e < VEC; ++e)
            if (v[e] > m[e]) { m[e] = v[e]; arg[e] = t; }
    }
    float g[VEC];
    Vec<T, VEC>::load(dy + ov * ldg + cv * VEC, g);
    for (int t = 0; t < 8; ++t) {
        int i = t >> 2, j = (t >> 1) & 1, k = t & 1;
        int64_t iv = (((int64_t)n * D + 2 * d + i) * H + 2 * h + j) * W + 2 * w + k;
        float o[VEC];
        if (add) Vec<T, VEC>::load(add + iv * lda + cv * VEC, o);
        else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) o[e] = 0.f;
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) o[e] += (arg[e] == t) ? g[e] : 0.f;
        Vec<T, VEC>::store(dx + iv * ldo + cv * VEC, o);
    }
}

}  // namespace lamp

using namespace lamp;


static lamp_status pool_shapes(const lamp_tensor_desc* xd, const lamp_tensor_desc* yd) {
    if (!desc_ok(xd) || !desc_ok(yd)) return LAMP_ERR_SHAPE;
    if ((xd->d & 1) || (xd->h & 1) || (xd->w & 1)) return LAMP_ERR_SHAPE;
    if (yd->n != xd->n || yd->d * 2 != xd->d || yd->h * 2 != xd->h || yd->w * 2 != xd->w || yd->c != xd->c)
        return LAMP_ERR_SHAPE;
    if (xd->dtype != yd->dtype) return LAMP_ERR_DTYPE;
    return LAMP_OK;
}

// InstanceNorm + ReLU of a raw conv output and the max-pool of the result in one pass: writes the activated
// tensor (yfull, channel stride ldyf) and its pooled version.  Same arithmetic and rounding as the two
// separate passes; one read of the full-resolution tensor less.
lamp_status lamp::inorm_relu_maxpool2(const lamp_tensor_desc* xd, const void* z, const lamp_norm_in* xnorm, void* yfull, int ldyf,
                                      const lamp_tensor_desc* yd, void* y, hipStream_t s) {
    if (!xd || !yd || !z || !y || !yfull || !xnorm || !xnorm->mean_rstd) return LAMP_ERR_NULL;
    lamp_status st = pool_shapes(xd, yd);
    if (st != LAMP_OK) return st;
    if ((st = norm_ok(xnorm, xd)) != LAMP_OK) return st;
    if (xnorm->c_norm != xd->c) return LAMP_ERR_SHAPE;
    const int vec = pick_vec(xd->dtype, xd->c, {xd->ldc, yd->ldc, ldyf}, {z, y, yfull});
    NormIn nm = make_norm(xnorm);
    LAMP_DISPATCH_TV(xd->dtype, vec, {
        int64_t total = nvox(yd) * (xd->c / VEC);
        hipLaunchKernelGGL((maxpool2_fwd_kernel<T, VEC>), dim3(cdiv(total, 256)), dim3(256), 0, s, (const T*)z, xd->ldc, nm,
                           (T*)y, yd->ldc, yd->n, yd->d, yd->h, yd->w, xd->c, (T*)yfull, ldyf);
    });
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}

extern "C" lamp_status lamp_maxpool2_fwd(const lamp_tensor_desc* xd, const void* x, const lamp_norm_in* xnorm,
                                         const lamp_tensor_desc* yd, void* y, void* stream) {
    if (!xd || !yd || !x || !y) return LAMP_ERR_NULL;
    lamp_status st = pool_shapes(xd, yd);
    if (st != LAMP_OK) return st;
    if ((st = norm_ok(xnorm, xd)) != LAMP_OK) return st;
    const int vec = pick_vec(xd->dtype, xd->c, {xd->ldc, yd->ldc}, {x, y});
    NormIn nm = make_norm(xnorm);
    LAMP_DISPATCH_TV(xd->dtype, vec, {
        int64_t total = nvox(yd) * (xd->c / VEC);
        hipLaunchKernelGGL((maxpool2_fwd_kernel<T, VEC>), dim3(cdiv(total, 256)), dim3(256), 0, (hipStream_t)stream,
                           (const T*)x, xd->ldc, nm, (T*)y, yd->ldc, yd->n, yd->d, yd->h, yd->w, xd->c);
    });
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}

extern "C" lamp_status lamp_maxpool2_bwd(const lamp_tensor_desc* xd, const void* x, const lamp_norm_in* xnorm,
                                         const lamp_tensor_desc* dyd, const void* dy, const lamp_tensor_desc* addd,
                                         const void* add, const lamp_tensor_desc* dxd, void* dx, void* stream) {
    if (!xd || !dyd || !dxd || !x || !dy || !dx) return LAMP_ERR_NULL;
    lamp_status st = pool_shapes(xd, dyd);
    if (st != LAMP_OK) return st;
    if (!desc_ok(dxd) || !same_space(xd, dxd) || dxd->c != xd->c) return LAMP_ERR_SHAPE;
    if (dxd->dtype != xd->dtype) return LAMP_ERR_DTYPE;
    int lda = 0;
    if (add) {
        if (!addd) return LAMP_ERR_NULL;
        if (!desc_ok(addd) || !same_space(xd, addd) || addd->c != xd->c) return LAMP_ERR_SHAPE;
        if (addd->dtype != xd->dtype) return LAMP_ERR_DTYPE;
        lda = addd->ldc;
    }
    if ((st = norm_ok(xnorm, xd)) != LAMP_OK) return st;
    const int vec = pick_vec(xd->dtype, xd->c, {xd->ldc, dyd->ldc, dxd->ldc, add ? lda : xd->ldc}, {x, dy, dx, add});
    NormIn nm = make_norm(xnorm);
    LAMP_DISPATCH_TV(xd->dtype, vec, {
        int64_t total = nvox(dyd) * (xd->c / VEC);
        hipLaunchKernelGGL((maxpool2_bwd_kernel<T, VEC>), dim3(cdiv(total, 256)), dim3(256), 0, (hipStream_t)stream,
                           (const T*)x, xd->ldc, nm, (const T*)dy, dyd->ldc, (const T*)add, lda, (T*)dx, dxd->ldc,
                           dyd->n, dyd->d, dyd->h, dyd->w, xd->c);
    });
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}
