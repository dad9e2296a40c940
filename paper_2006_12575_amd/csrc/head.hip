// 1x1x1 head, softmax and cross entropy (forward and backward).  One thread per voxel; the
// op is bound by reading the activations and writing the fp32 logits.
#include "internal.h"
#include "vec.h"

namespace lamp {

static const int kMaxClasses = 16;

// KM: compile-time bound on the class count (4, 8 or 16).
// MODE 0: logits only.  MODE 1: + loss partials, dlogits, dx.
template <typename T, int VEC, int MODE, int KM>
__global__ __launch_bounds__(256) void head_kernel(const T* __restrict__ x, int ldx, NormIn nm, const T* __restrict__ wh,
                                                   const float* __restrict__ bh, int K, int C, int64_t Vs, int64_t Vtot,
                                                   const int32_t* __restrict__ labels, float* __restrict__ logits,
                                                   float* __restrict__ dlogits, T* __restrict__ dx, int lddx,
                                                   float* __restrict__ loss_part) {
    extern __shared__ float wsh[];  // [K][C]
    __shared__ float red[256];
    for (int i = threadIdx.x; i < K * C; i += 256) wsh[i] = io<T>::ld(wh + i);
    __syncthreads();
    float lsum = 0.f;
    const float invV = 1.0f / (float)Vtot;
    for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < Vtot; v += (int64_t)gridDim.x * 256) {
        const int n = (int)(v / Vs);
        float acc[KM];
#pragma unroll
        for (int k = 0; k < KM; ++k) acc[k] = (k < K && bh) ? bh[k] : 0.f;
        const T* xp = x + v * ldx;
        for (int c0 = 0; c0 < C; c0 += VEC) {
            float xv[VEC];
            load_norm_vec<T, VEC>(xp + c0, nm, n, c0, xv);
#pragma unroll
            for (int i = 0; i < VEC; ++i)
#pragma unroll
                for (int k = 0; k < KM; ++k)
                    if (k < K) acc[k] = fmaf(xv[i], wsh[k * C + c0 + i], acc[k]);
        }
        if (logits) {
#pragma unroll
            for (int k = 0; k < KM; ++k)
                if (k < K) logits[v * K + k] = acc[k];
        }
        if (MODE == 1) {
            float m = acc[0];
#pragma unroll
            for (int k = 1; k < KM; ++k)
                if (k < K) m = acc[k] > m ? acc[k] : m;
            float se = 0.f;
#pragma unroll
            for (int k = 0; k < KM; ++k)
                if (k < K) se += expf(acc[k] - m);
            const float lse = m + logf(se);
            const int lab = labels[v];
            float ll = 0.f;
#pragma unroll
            for (int k = 0; k < KM; ++k) {
                if (k < K) {
                    if (k == lab) ll = acc[k];
                    float p = expf(acc[k] - lse);
                    acc[k] = (p - (k == lab ? 1.f : 0.f)) * invV;
                    dlogits[v * K + k] = acc[k];
                }
            }
            lsum += (lse - ll) * invV;
            if (dx) {
                for (int c0 = 0; c0 < C; c0 += VEC) {
                    float g[VEC];
#pragma unroll
                    for (int i = 0; i < VEC; ++i) {
                        g[i] = 0.f;
#pragma unroll
                        for (int k = 0; k < KM; ++k)
                            if (k < K) g[i] = fmaf(acc[k], wsh[k * C + c0 + i], g[i]);
                    }
                    Vec<T, VEC>::store(dx + v * lddx + c0, g);
                }
            }
        }
    }
    if (MODE == 1) {
        red[threadIdx.x] = lsum;
        __syncthreads();
        for (int off = 128; off > 0; off >>= 1) {
            if (threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
            __syncthreads();
        }
        if (threadIdx.x == 0) loss_part[blockIdx.x] = red[0];
    }
}

// part[s][k*C + c] = sum over the voxels of split s of dlogits[v][k] * X[v][c].  Threads side by
// side cover the channels of one voxel row (coalesced), 256/C voxel rows are in flight per block and
// every thread keeps K sums; the row lanes are then added in order through LDS.
template <typename T, int KM>
__global__ __launch_bounds__(256) void head_wgrad_kernel(const T* __restrict__ x, int ldx, NormIn nm,
                                                         const float* __restrict__ dlogits, int K, int C, int64_t Vs,
                                                         int64_t Vtot, int64_t vps, float* __restrict__ part) {
    __shared__ float red[KM * 256];
    const int cthreads = C < 256 ? C : 256;
    const int rl = 256 / cthreads;
    const int cl = threadIdx.x % cthreads, r0 = threadIdx.x / cthreads;
    const int c = blockIdx.y * 256 + cl;
    int64_t v0 = (int64_t)blockIdx.x * vps, v1 = v0 + vps;
    if (v1 > Vtot) v1 = Vtot;
    float acc[KM];
#pragma unroll
    for (int k = 0; k < KM; ++k) acc[k] = 0.f;
    if (r0 < rl && c < C)
        for (int64_t v = v0 + r0; v < v1; v += rl) {
            const float xv = load_norm(x + v * ldx + c, nm, (int)(v / Vs), c);
            const float* dl = dlogits + v * K;
#pragma unroll
            for (int k = 0; k < KM; ++k)
                if (k < K) acc[k] = fmaf(dl[k], xv, acc[k]);
        }
#pragma unroll
    for (int k = 0; k < KM; ++k)
        if (k < K) red[k * 256 + threadIdx.x] = acc[k];
    __syncthreads();
    if (r0 == 0 && c < C)
        for (int k = 0; k < K; ++k) {
            float t = 0.f;
            for (int r = 0; r < rl; ++r) t += red[k * 256 + r * cthreads + cl];
            part[(int64_t)blockIdx.x * K * C + (int64_t)k * C + c] = t;
        }
}

static int head_blocks(int64_t V) {
    int64_t b = (V + 255) / 256;
    return (int)(b > 2048 ? 2048 : b);
}
static int head_splits(int64_t V) {
    int64_t s = (V + 511) / 512;
    return (int)(s > 4096 ? 4096 : (s < 1 ? 1 : s));
}

static lamp_status head_check(const lamp_tensor_desc* xd, const void* x, const void* wh, int classes) {
    if (!xd || !x || !wh) return LAMP_ERR_NULL;
    if (!desc_ok(xd) || classes < 1 || classes > kMaxClasses) return LAMP_ERR_SHAPE;
    if ((size_t)classes * xd->c * sizeof(float) > 48 * 1024) return LAMP_ERR_UNSUPPORTED;
    return LAMP_OK;
}

}  // namespace lamp

using namespace lamp;

#define LAMP_DISPATCH_KM(k, BODY)                      \
    do {                                               \
        if ((k) <= 4) { constexpr int KM = 4; BODY }   \
        else if ((k) <= 8) { constexpr int KM = 8; BODY } \
        else { constexpr int KM = 16; BODY }           \
    } while (0)

extern "C" lamp_status lamp_head_fwd(const lamp_tensor_desc* xd, const void* x, const lamp_norm_in* xnorm, const void* wh,
                                     const float* bh, int classes, float* logits, void* stream) {
    lamp_status st = head_check(xd, x, wh, classes);
    if (st != LAMP_OK) return st;
    if (!logits) return LAMP_ERR_NULL;
    if ((st = norm_ok(xnorm, xd)) != LAMP_OK) return st;
    const int64_t Vs = (int64_t)xd->d * xd->h * xd->w, Vt = nvox(xd);
    const size_t shm = (size_t)classes * xd->c * sizeof(float);
    NormIn nm = make_norm(xnorm);
    const int vec = pick_vec(xd->dtype, xd->c, {xd->ldc}, {x});
    LAMP_DISPATCH_TV(xd->dtype, vec, {
        LAMP_DISPATCH_KM(classes, {
            hipLaunchKernelGGL((head_kernel<T, VEC, 0, KM>), dim3(head_blocks(Vt)), dim3(256), shm, (hipStream_t)stream,
                               (const T*)x, xd->ldc, nm, (const T*)wh, bh, classes, xd->c, Vs, Vt, nullptr, logits,
                               nullptr, (T*)nullptr, 0, nullptr);
        });
    });
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}

extern "C" size_t lamp_head_ce_workspace_bytes(const lamp_tensor_desc* xd, int classes) {
    if (!desc_ok(xd) || classes < 1) return 0;
    const int64_t Vt = nvox(xd);
    return align_up((size_t)Vt * classes * sizeof(float)) + align_up((size_t)head_blocks(Vt) * sizeof(float)) +
           align_up((size_t)head_splits(Vt) * classes * xd->c * sizeof(float)) + colsum_ws_bytes(Vt, classes);
}

extern "C" lamp_status lamp_head_ce(const lamp_tensor_desc* xd, const void* x, const lamp_norm_in* xnorm, const void* wh,
                                    const float* bh, int classes, const int32_t* labels, float* logits, float* loss,
                                    const lamp_tensor_desc* dxd, void* dx, float* dwh, float* dbh, float beta, void* ws,
                                    size_t ws_bytes, void* stream) {
    lamp_status st = head_check(xd, x, wh, classes);
    if (st != LAMP_OK) return st;
    if (!labels || !loss) return LAMP_ERR_NULL;
    if ((st = norm_ok(xnorm, xd)) != LAMP_OK) return st;
    if (beta != 0.f && beta != 1.f) return LAMP_ERR_SHAPE;
    int lddx = 0;
    if (dx) {
        if (!dxd) return LAMP_ERR_NULL;
        if (!desc_ok(dxd) || !same_space(xd, dxd) || dxd->c != xd->c) return LAMP_ERR_SHAPE;
        if (dxd->dtype != xd->dtype) return LAMP_ERR_DTYPE;
        lddx = dxd->ldc;
    }
    if (!ws || ws_bytes < lamp_head_ce_workspace_bytes(xd, classes)) return LAMP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int64_t Vs = (int64_t)xd->d * xd->h * xd->w, Vt = nvox(xd);
    const int K = classes, C = xd->c;
    Carver cv(ws, ws_bytes);
    float* dlogits = (float*)cv.take((size_t)Vt * K * sizeof(float));
    const int nb = head_blocks(Vt);
    float* lpart = (float*)cv.take((size_t)nb * sizeof(float));
    const int S = head_splits(Vt);
    float* wpart = (float*)cv.take((size_t)S * K * C * sizeof(float));
    const size_t csb = colsum_ws_bytes(Vt, K);
    void* csws = cv.take(csb);
    if (!cv.ok()) return LAMP_ERR_WORKSPACE;
    const size_t shm = (size_t)K * C * sizeof(float);
    NormIn nm = make_norm(xnorm);
    const int vec = pick_vec(xd->dtype, C, {xd->ldc, lddx}, {x, dx});
    LAMP_DISPATCH_TV(xd->dtype, vec, {
        LAMP_DISPATCH_KM(K, {
            hipLaunchKernelGGL((head_kernel<T, VEC, 1, KM>), dim3(nb), dim3(256), shm, s, (const T*)x, xd->ldc, nm,
                               (const T*)wh, bh, K, C, Vs, Vt, labels, logits, dlogits, (T*)dx, lddx, lpart);
        });
    });
    LAMP_CHECK_LAUNCH();
    if ((st = launch_reduce_partials(lpart, nb, 1, loss, 0.f, s)) != LAMP_OK) return st;
    if (dwh) {
        const int64_t vps = (Vt + S - 1) / S;
        dim3 grid(S, cdiv(C, 256));
        LAMP_DISPATCH_KM(K, {
            if (xd->dtype == LAMP_BF16)
                hipLaunchKernelGGL((head_wgrad_kernel<bf16_t, KM>), grid, dim3(256), 0, s, (const bf16_t*)x, xd->ldc, nm,
                                   dlogits, K, C, Vs, Vt, vps, wpart);
            else
                hipLaunchKernelGGL((head_wgrad_kernel<float, KM>), grid, dim3(256), 0, s, (const float*)x, xd->ldc, nm,
                                   dlogits, K, C, Vs, Vt, vps, wpart);
        });
        LAMP_CHECK_LAUNCH();
        if ((st = launch_reduce_partials(wpart, S, (int64_t)K * C, dwh, beta, s)) != LAMP_OK) return st;
    }
    if (dbh) {
        if ((st = launch_colsum(dlogits, LAMP_F32, Vt, K, K, dbh, beta, csws, csb, s)) != LAMP_OK) return st;
    }
    return LAMP_OK;
}
