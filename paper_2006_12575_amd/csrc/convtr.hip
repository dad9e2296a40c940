// 2x2x2 stride-2 transposed convolution (decoder upsampling), forward and backward.
// Each output voxel depends on exactly one input voxel and one of the 8 taps, so the op is a
// [V_in, Ci] x [Ci, 8*Co] product scattered to the 2x2x2 sub-positions; at the U-Net's upper
// levels it is bound by writing the output, which goes straight into the concat buffer.
#include "internal.h"

namespace lamp {

template <typename T>
__global__ __launch_bounds__(256) void convtr_fwd_kernel(const T* __restrict__ x, int ldx, NormIn nm,
                                                         const T* __restrict__ wt, const float* __restrict__ bias,
                                                         T* __restrict__ y, int ldy, int N, int D, int H, int W, int Ci,
                                                         int Co) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = (int64_t)N * 8 * D * H * W * Co;
    if (idx >= total) return;
    const int co = (int)(idx % Co);
    int64_t ov = idx / Co;
    const int ow = (int)(ov % (2 * W));
    int64_t r = ov / (2 * W);
    const int oh = (int)(r % (2 * H));
    r /= (2 * H);
    const int od = (int)(r % (2 * D));
    const int n = (int)(r / (2 * D));
    const int tap = ((od & 1) * 2 + (oh & 1)) * 2 + (ow & 1);
    const T* xp = x + ((((int64_t)n * D + (od >> 1)) * H + (oh >> 1)) * W + (ow >> 1)) * ldx;
    const T* wp = wt + (int64_t)tap * Co + co;
    float acc = bias ? bias[co] : 0.f;
    for (int ci = 0; ci < Ci; ++ci) acc = fmaf(load_norm(xp + ci, nm, n, ci), io<T>::ld(wp + (int64_t)ci * 8 * Co), acc);
    io<T>::st(y + ov * ldy + co, acc);
}

template <typename T>
__global__ __launch_bounds__(256) void convtr_dgrad_kernel(const T* __restrict__ dy, int ldg, const T* __restrict__ wt,
                                                           T* __restrict__ dx, int ldo, int N, int D, int H, int W,
                                                           int Ci, int Co) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = (int64_t)N * D * H * W * Ci;
    if (idx >= total) return;
    const int ci = (int)(idx % Ci);
    int64_t iv = idx / Ci;
    const int w = (int)(iv % W);
    int64_t r = iv / W;
    const int h = (int)(r % H);
    r /= H;
    const int d = (int)(r % D);
    const int n = (int)(r / D);
    float acc = 0.f;
    for (int tap = 0; tap < 8; ++tap) {
        int i = tap >> 2, j = (tap >> 1) & 1, k = tap & 1;
        const T* gp = dy + ((((int64_t)n * 2 * D + 2 * d + i) * 2 * H + 2 * h + j) * 2 * W + 2 * w + k) * ldg;
        const T* wp = wt + ((int64_t)ci * 8 + tap) * Co;
        for (int co = 0; co < Co; ++co) acc = fmaf(io<T>::ld(gp + co), io<T>::ld(wp + co), acc);
    }
    io<T>::st(dx + iv * ldo + ci, acc);
}

// part[s][o], o = (ci*8 + tap)*Co + co, over the input voxels of split s.
template <typename T>
__global__ __launch_bounds__(256) void convtr_wgrad_kernel(const T* __restrict__ x, int ldx, NormIn nm,
                                                           const T* __restrict__ dy, int ldg, float* __restrict__ part,
                                                           int N, int D, int H, int W, int Ci, int Co, int64_t vps) {
    const int64_t O = (int64_t)Ci * 8 * Co;
    const int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (o >= O) return;
    const int co = (int)(o % Co);
    const int tap = (int)((o / Co) % 8);
    const int ci = (int)(o / ((int64_t)8 * Co));
    const int i = tap >> 2, j = (tap >> 1) & 1, k = tap & 1;
    const int64_t total = (int64_t)N * D * H * W;
    int64_t v0 = (int64_t)blockIdx.y * vps, v1 = v0 + vps;
    if (v1 > total) v1 = total;
    int w = (int)(v0 % W);
    int64_t r = v0 / W;
    int h = (int)(r % H);
    r /= H;
    int d = (int)(r % D);
    int n = (int)(r / D);
    float acc = 0.f;
    for (int64_t v = v0; v < v1; ++v) {
        const T* gp = dy + ((((int64_t)n * 2 * D + 2 * d + i) * 2 * H + 2 * h + j) * 2 * W + 2 * w + k) * ldg + co;
        acc = fmaf(load_norm(x + v * ldx + ci, nm, n, ci), io<T>::ld(gp), acc);
        if (++w == W) { w = 0; if (++h == H) { h = 0; if (++d == D) { d = 0; ++n; } } }
    }
    part[(int64_t)blockIdx.y * O + o] = acc;
}

static int convtr_splits(int64_t V, int64_t O) {
    int64_t s = (V + 127) / 128;
    int64_t cap = (int64_t)(32u << 20) / (O * 4);
    if (cap < 1) cap = 1;
    if (s > cap) s = cap;
    if (s > 4096) s = 4096;
    if (s < 1) s = 1;
    return (int)s;
}

static lamp_status convtr_shapes(const lamp_tensor_desc* xd, const lamp_tensor_desc* yd) {
    if (!desc_ok(xd) || !desc_ok(yd)) return LAMP_ERR_SHAPE;
    if (yd->n != xd->n || yd->d != 2 * xd->d || yd->h != 2 * xd->h || yd->w != 2 * xd->w) return LAMP_ERR_SHAPE;
    if (xd->dtype != yd->dtype) return LAMP_ERR_DTYPE;
    return LAMP_OK;
}

}  // namespace lamp

using namespace lamp;

extern "C" size_t lamp_convtr3d_workspace_bytes(const lamp_tensor_desc* xd, const lamp_tensor_desc* yd) {
    if (!desc_ok(xd) || !desc_ok(yd)) return 0;
    return mfma_convtr_ws_bytes(xd, yd);
}

extern "C" lamp_status lamp_convtr3d(const lamp_tensor_desc* xd, const void* x, const lamp_norm_in* xnorm, const void* wt,
                                     const float* bias, const lamp_tensor_desc* yd, void* y, void* ws, size_t ws_bytes,
                                     void* stream) {
    if (!xd || !yd || !x || !wt || !y) return LAMP_ERR_NULL;
    lamp_status st = convtr_shapes(xd, yd);
    if (st != LAMP_OK) return st;
    if ((st = norm_ok(xnorm, xd)) != LAMP_OK) return st;
    if (ws_bytes < lamp_convtr3d_workspace_bytes(xd, yd) || (ws_bytes && !ws)) return LAMP_ERR_WORKSPACE;
    if (mfma_convtr_supported(xd, yd, xnorm) && aligned16(x) && aligned16(ws) && ((((uintptr_t)y) & 7u) == 0))
        return mfma_convtr_fwd(xd, x, wt, bias, yd, y, ws, ws_bytes, (hipStream_t)stream);
    NormIn nm = make_norm(xnorm);
    const int64_t total = nvox(yd) * yd->c;
    if (xd->dtype == LAMP_BF16)
        hipLaunchKernelGGL((convtr_fwd_kernel<bf16_t>), dim3(cdiv(total, 256)), dim3(256), 0, (hipStream_t)stream,
                           (const bf16_t*)x, xd->ldc, nm, (const bf16_t*)wt, bias, (bf16_t*)y, yd->ldc, xd->n, xd->d,
                           xd->h, xd->w, xd->c, yd->c);
    else
        hipLaunchKernelGGL((convtr_fwd_kernel<float>), dim3(cdiv(total, 256)), dim3(256), 0, (hipStream_t)stream,
                           (const float*)x, xd->ldc, nm, (const float*)wt, bias, (float*)y, yd->ldc, xd->n, xd->d, xd->h,
                           xd->w, xd->c, yd->c);
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}

extern "C" size_t lamp_convtr3d_bwd_workspace_bytes(const lamp_tensor_desc* xd, const lamp_tensor_desc* dyd) {
    if (!desc_ok(xd) || !desc_ok(dyd)) return 0;
    const int64_t O = (int64_t)xd->c * 8 * dyd->c;
    size_t a = align_up((size_t)convtr_splits(nvox(xd), O) * O * sizeof(float));
    const size_t b = mfma_convtr_wgrad_ws_bytes(xd, dyd);
    if (b > a) a = align_up(b);
    return a + colsum_ws_bytes(nvox(dyd), dyd->c);
}

extern "C" lamp_status lamp_convtr3d_bwd(const lamp_tensor_desc* xd, const void* x, const lamp_norm_in* xnorm,
                                         const void* wt, const lamp_tensor_desc* dyd, const void* dy,
                                         const lamp_tensor_desc* dxd, void* dx, float* dwt, float* dbias, float beta,
                                         void* ws, size_t ws_bytes, void* stream) {
    if (!xd || !dyd || !x || !wt || !dy) return LAMP_ERR_NULL;
    lamp_status st = convtr_shapes(xd, dyd);
    if (st != LAMP_OK) return st;
    if ((st = norm_ok(xnorm, xd)) != LAMP_OK) return st;
    if (beta != 0.f && beta != 1.f) return LAMP_ERR_SHAPE;
    if (dx) {
        if (!dxd) return LAMP_ERR_NULL;
        if (!desc_ok(dxd) || !same_space(xd, dxd) || dxd->c != xd->c) return LAMP_ERR_SHAPE;
        if (dxd->dtype != xd->dtype) return LAMP_ERR_DTYPE;
    }
    if ((dwt || dbias) && (!ws || ws_bytes < lamp_convtr3d_bwd_workspace_bytes(xd, dyd))) return LAMP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int Ci = xd->c, Co = dyd->c;
    if (dx && mfma_convtr_dgrad_supported(xd, dyd, dxd) && aligned16(dy) && aligned16(wt) && ((((uintptr_t)dx) & 7u) == 0)) {
        if ((st = mfma_convtr_dgrad(xd, wt, dyd, dy, dxd, dx, s)) != LAMP_OK) return st;
    } else if (dx) {
        const int64_t total = nvox(xd) * Ci;
        if (xd->dtype == LAMP_BF16)
            hipLaunchKernelGGL((convtr_dgrad_kernel<bf16_t>), dim3(cdiv(total, 256)), dim3(256), 0, s, (const bf16_t*)dy,
                               dyd->ldc, (const bf16_t*)wt, (bf16_t*)dx, dxd->ldc, xd->n, xd->d, xd->h, xd->w, Ci, Co);
        else
            hipLaunchKernelGGL((convtr_dgrad_kernel<float>), dim3(cdiv(total, 256)), dim3(256), 0, s, (const float*)dy,
                               dyd->ldc, (const float*)wt, (float*)dx, dxd->ldc, xd->n, xd->d, xd->h, xd->w, Ci, Co);
        LAMP_CHECK_LAUNCH();
    }
    const int64_t O = (int64_t)Ci * 8 * Co;
    const size_t csb = colsum_ws_bytes(nvox(dyd), Co);
    const size_t pbytes = lamp_convtr3d_bwd_workspace_bytes(xd, dyd) - csb;
    if (dwt && mfma_convtr_wgrad_supported(xd, dyd, xnorm) && aligned16(x) && aligned16(dy) && aligned16(ws)) {
        if ((st = mfma_convtr_wgrad(xd, x, dyd, dy, dwt, beta, ws, pbytes, s)) != LAMP_OK) return st;
    } else if (dwt) {
        const int64_t V = nvox(xd);
        const int S = convtr_splits(V, O);
        const int64_t vps = (V + S - 1) / S;
        float* part = (float*)ws;
        NormIn nm = make_norm(xnorm);
        dim3 grid(cdiv(O, 256), S);
        if (xd->dtype == LAMP_BF16)
            hipLaunchKernelGGL((convtr_wgrad_kernel<bf16_t>), grid, dim3(256), 0, s, (const bf16_t*)x, xd->ldc, nm,
                               (const bf16_t*)dy, dyd->ldc, part, xd->n, xd->d, xd->h, xd->w, Ci, Co, vps);
        else
            hipLaunchKernelGGL((convtr_wgrad_kernel<float>), grid, dim3(256), 0, s, (const float*)x, xd->ldc, nm,
                               (const float*)dy, dyd->ldc, part, xd->n, xd->d, xd->h, xd->w, Ci, Co, vps);
        LAMP_CHECK_LAUNCH();
        st = launch_reduce_partials(part, S, O, dwt, beta, s);
        if (st != LAMP_OK) return st;
    }
    if (dbias) {
        st = launch_colsum(dy, dyd->dtype, nvox(dyd), Co, dyd->ldc, dbias, beta, (char*)ws + pbytes,
                           colsum_ws_bytes(nvox(dyd), Co), s);
        if (st != LAMP_OK) return st;
    }
    return LAMP_OK;
}
