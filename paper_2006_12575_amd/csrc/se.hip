// Squeeze-and-excitation on top of InstanceNorm + ReLU (the SEU-Net variant the paper names in Sec. 1
// through its citations):
//   a = max(0, gamma*zhat + beta)         (never stored)
//   m[n,c] = mean_v a                     squeeze
//   h = max(0, W1 m + b1), e = sigmoid(W2 h + b2)   excitation, W1 [Cr,C], W2 [C,Cr], fp32
//   y = a * e[n,c] (+ residual)
// Everything here is bandwidth-bound: forward = one read of z for the squeeze, one read of z (and of the
// residual) + one write of y for the scale; backward = one read of (dy, z) for three per-(n,c) sums from
// which, with two sums the forward keeps, both the gate's gradient and the two InstanceNorm-backward
// sums follow, then one read of (dy, z) + one write of dz for the apply.  All reductions are two-stage
// in a fixed order (fp32 partials per row chunk, fp64 across chunks).
#include "internal.h"
#include "vec.h"

namespace lamp {

// Three sums per (n,c) over a chunk of rows (mask = [u > 0]):
// MODE 0 (forward):  sum a, sum mask, sum mask*zhat        (the last two are kept for the backward)
// MODE 1 (backward): sum dy*a, sum dy*mask, sum dy*mask*zhat
// partial[((n*chunks + chunk)*C + c)*3 + k]
template <typename T, int VEC, int MODE>
__global__ __launch_bounds__(256) void se_partial_kernel(const T* __restrict__ dy, int ldg, const T* __restrict__ z, int ldz,
                                                         int64_t V, int C, int cthreads, int rl, int rows_per_chunk,
                                                         const float* __restrict__ stats, const float* __restrict__ gamma,
                                                         const float* __restrict__ beta, float* __restrict__ partial) {
    constexpr int K = 3;
    __shared__ float red[K][256 * VEC];
    const int tid = threadIdx.x;
    const int cl = tid % cthreads, r0 = tid / cthreads;
    const int cv = blockIdx.z * 256 + cl;
    const int chunk = blockIdx.x, n = blockIdx.y, chunks = gridDim.x;
    const int64_t rbeg = (int64_t)chunk * rows_per_chunk;
    int64_t rend = rbeg + rows_per_chunk;
    if (rend > V) rend = V;
    float s[K][VEC];
#pragma unroll
    for (int k = 0; k < K; ++k)
#pragma unroll
        for (int i = 0; i < VEC; ++i) s[k][i] = 0.f;
    if (r0 < rl && cv * VEC < C) {
        NormIn nm{stats, gamma, beta, C, 1};
        float a[VEC], b[VEC], mean[VEC], rstd[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            norm_coeffs(nm, n, cv * VEC + i, a[i], b[i]);
            mean[i] = stats[((size_t)n * C + cv * VEC + i) * 2];
            rstd[i] = stats[((size_t)n * C + cv * VEC + i) * 2 + 1];
        }
        const T* zb = z + ((int64_t)n * V) * ldz + (int64_t)cv * VEC;
        const T* gb = MODE == 1 ? dy + ((int64_t)n * V) * ldg + (int64_t)cv * VEC : nullptr;
        auto add_row = [&](const float (&v)[VEC], const float (&g)[VEC]) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                const float u = norm_u(v[i], a[i], b[i]);
                const bool on = u > 0.f;
                const float zh = (v[i] - mean[i]) * rstd[i];
                if (MODE == 0) {
                    s[0][i] += on ? u : 0.f;
                    s[1][i] += on ? 1.f : 0.f;
                    s[2][i] += on ? zh : 0.f;
                } else {
                    const float gg = on ? g[i] : 0.f;
                    s[0][i] = fmaf(gg, u, s[0][i]);
                    s[1][i] += gg;
                    s[2][i] = fmaf(gg, zh, s[2][i]);
                }
            }
        };
        int64_t r = rbeg + r0;
        // four rows in flight; the additions keep the row order
        for (; r + 3 * (int64_t)rl < rend; r += 4 * (int64_t)rl) {
            float v[4][VEC], g[4][VEC];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                Vec<T, VEC>::load(zb + (r + u * (int64_t)rl) * ldz, v[u]);
                if (MODE == 1) Vec<T, VEC>::load(gb + (r + u * (int64_t)rl) * ldg, g[u]);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) add_row(v[u], g[u]);
        }
        for (; r < rend; r += rl) {
            float v[VEC], g[VEC];
            Vec<T, VEC>::load(zb + r * ldz, v);
            if (MODE == 1) Vec<T, VEC>::load(gb + r * ldg, g);
            add_row(v, g);
        }
    }
#pragma unroll
    for (int k = 0; k < K; ++k)
#pragma unroll
        for (int i = 0; i < VEC; ++i) red[k][tid * VEC + i] = s[k][i];
    __syncthreads();
    if (r0 == 0 && cv * VEC < C) {
        for (int i = 0; i < VEC; ++i) {
            const size_t o = (((size_t)n * chunks + chunk) * C + (size_t)cv * VEC + i) * K;
            for (int k = 0; k < K; ++k) {
                float t = 0.f;
                for (int r = 0; r < rl; ++r) t += red[k][(r * cthreads + cl) * VEC + i];
                partial[o + k] = t;
            }
        }
    }
}

// sums[(n*C + c)*K + k] = sum over the chunks, fp64, fixed order.
template <int K>
__global__ __launch_bounds__(256) void se_finalize_kernel(const float* __restrict__ partial, int parts, int C,
                                                          float* __restrict__ sums) {
    __shared__ double sh[4][K];
    const int c = blockIdx.x, n = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const float* pp = partial + ((size_t)n * parts * C + c) * K;
    double s[K];
#pragma unroll
    for (int k = 0; k < K; ++k) s[k] = 0.0;
    for (int p = tid; p < parts; p += 256)
#pragma unroll
        for (int k = 0; k < K; ++k) s[k] += (double)pp[(size_t)p * C * K + k];
#pragma unroll
    for (int k = 0; k < K; ++k)
        for (int off = 32; off > 0; off >>= 1) s[k] += __shfl_down(s[k], off);
    if (lane == 0)
#pragma unroll
        for (int k = 0; k < K; ++k) sh[wv][k] = s[k];
    __syncthreads();
    if (tid == 0)
#pragma unroll
        for (int k = 0; k < K; ++k) sums[((size_t)n * C + c) * K + k] = (float)(sh[0][k] + sh[1][k] + sh[2][k] + sh[3][k]);
}

// One workgroup per sample.  save[n] = { m[C], e[C], h[Cr], sum mask [C], sum mask*zhat [C] }; a3[n][c][3] as
// written by the MODE 0 sums.
__global__ __launch_bounds__(256) void se_gate_kernel(const float* __restrict__ a3, float invV, int C, int Cr,
                                                      const float* __restrict__ w1, const float* __restrict__ b1,
                                                      const float* __restrict__ w2, const float* __restrict__ b2,
                                                      float* __restrict__ save) {
    extern __shared__ float sm[];   // m[C], h[Cr]
    float* m = sm;
    float* h = sm + C;
    const int n = blockIdx.x, tid = threadIdx.x;
    float* sv = save + (size_t)n * (4 * C + Cr);
    for (int c = tid; c < C; c += 256) {
        const float* q = a3 + ((size_t)n * C + c) * 3;
        const float v = q[0] * invV;
        m[c] = v;
        sv[c] = v;
        sv[2 * C + Cr + c] = q[1];
        sv[3 * C + Cr + c] = q[2];
    }
    __syncthreads();
    for (int j = tid; j < Cr; j += 256) {
        float t = b1 ? b1[j] : 0.f;
        for (int c = 0; c < C; ++c) t = fmaf(w1[(size_t)j * C + c], m[c], t);
        t = t > 0.f ? t : 0.f;
        h[j] = t;
        sv[2 * C + j] = t;
    }
    __syncthreads();
    for (int c = tid; c < C; c += 256) {
        float t = b2 ? b2[c] : 0.f;
        for (int j = 0; j < Cr; ++j) t = fmaf(w2[(size_t)c * Cr + j], h[j], t);
        sv[C + c] = 1.0f / (1.0f + expf(-t));
    }
}

template <typename T, int VEC, bool RES>
__global__ __launch_bounds__(256) void se_apply_kernel(const T* __restrict__ z, int ldz, const T* __restrict__ res, int ldr,
                                                       T* __restrict__ y, int ldy, int64_t V, int C, int Cr, int cthreads,
                                                       int rl, const float* __restrict__ stats,
                                                       const float* __restrict__ gamma, const float* __restrict__ beta,
                                                       const float* __restrict__ save) {
    const int tid = threadIdx.x;
    const int cl = tid % cthreads, r0 = tid / cthreads;
    const int cv = blockIdx.z * 256 + cl;
    const int n = blockIdx.y;
    if (r0 >= rl || cv * VEC >= C) return;
    NormIn nm{stats, gamma, beta, C, 1};
    float a[VEC], b[VEC], e[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        norm_coeffs(nm, n, cv * VEC + i, a[i], b[i]);
        e[i] = save[(size_t)n * (4 * C + Cr) + C + cv * VEC + i];
    }
    const T* zb = z + ((int64_t)n * V) * ldz + (int64_t)cv * VEC;
    const T* rb = RES ? res + ((int64_t)n * V) * ldr + (int64_t)cv * VEC : nullptr;
    T* yb = y + ((int64_t)n * V) * ldy + (int64_t)cv * VEC;
    for (int64_t r = (int64_t)blockIdx.x * rl + r0; r < V; r += (int64_t)gridDim.x * rl) {
        float v[VEC], q[VEC];
        Vec<T, VEC>::load(zb + r * ldz, v);
        if (RES) Vec<T, VEC>::load(rb + r * ldr, q);
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            const float u = norm_u(v[i], a[i], b[i]);
            const float act = u > 0.f ? u : 0.f;
            v[i] = RES ? fmaf(act, e[i], q[i]) : act * e[i];
        }
        Vec<T, VEC>::store(yb + r * ldy, v);
    }
}

// Backward of the gate, one workgroup per sample.  s3[n][c][3] as written by the MODE 1 sums.
// Writes dp2[n][C], dp1[n][Cr], dmv[n][C] = dm/V and the InstanceNorm-backward sums
// sums2[n][c] = (sum_v g*mask, sum_v g*mask*zhat) for g = dy*e + dm/V.
__global__ __launch_bounds__(256) void se_gate_bwd_kernel(const float* __restrict__ s3, float invV, int C, int Cr,
                                                          const float* __restrict__ w1, const float* __restrict__ w2,
                                                          const float* __restrict__ save, float* __restrict__ dp2,
                                                          float* __restrict__ dp1, float* __restrict__ dmv,
                                                          float* __restrict__ sums2) {
    extern __shared__ float sm[];   // p2[C], p1[Cr]
    float* p2 = sm;
    float* p1 = sm + C;
    const int n = blockIdx.x, tid = threadIdx.x;
    const float* sv = save + (size_t)n * (4 * C + Cr);
    for (int c = tid; c < C; c += 256) {
        const float e = sv[C + c];
        const float t = s3[((size_t)n * C + c) * 3] * e * (1.0f - e);
        p2[c] = t;
        dp2[(size_t)n * C + c] = t;
    }
    __syncthreads();
    for (int j = tid; j < Cr; j += 256) {
        float t = 0.f;
        for (int c = 0; c < C; ++c) t = fmaf(p2[c], w2[(size_t)c * Cr + j], t);
        t = sv[2 * C + j] > 0.f ? t : 0.f;
        p1[j] = t;
        dp1[(size_t)n * Cr + j] = t;
    }
    __syncthreads();
    for (int c = tid; c < C; c += 256) {
        float dm = 0.f;
        for (int j = 0; j < Cr; ++j) dm = fmaf(p1[j], w1[(size_t)j * C + c], dm);
        dm *= invV;
        const float e = sv[C + c];
        const float* q = s3 + ((size_t)n * C + c) * 3;
        dmv[(size_t)n * C + c] = dm;
        sums2[((size_t)n * C + c) * 2 + 0] = fmaf(e, q[1], dm * sv[2 * C + Cr + c]);
        sums2[((size_t)n * C + c) * 2 + 1] = fmaf(e, q[2], dm * sv[3 * C + Cr + c]);
    }
}

// Parameter gradients: sums over the samples in a fixed order.
// idx < C*Cr: dW2[c][j] and dW1[j][c] (idx = c*Cr + j); then db2 and db1 from the first C / Cr threads.
__global__ __launch_bounds__(256) void se_param_grad_kernel(const float* __restrict__ dp2, const float* __restrict__ dp1,
                                                            const float* __restrict__ save, int N, int C, int Cr,
                                                            float* __restrict__ dw1, float* __restrict__ db1,
                                                            float* __restrict__ dw2, float* __restrict__ db2, float acc) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    const int S = 4 * C + Cr;
    if (idx < C * Cr) {
        const int c = idx / Cr, j = idx % Cr;
        float t2 = 0.f, t1 = 0.f;
        for (int n = 0; n < N; ++n) {
            t2 = fmaf(dp2[(size_t)n * C + c], save[(size_t)n * S + 2 * C + j], t2);
            t1 = fmaf(dp1[(size_t)n * Cr + j], save[(size_t)n * S + c], t1);
        }
        if (dw2) dw2[(size_t)c * Cr + j] = (acc != 0.f ? acc * dw2[(size_t)c * Cr + j] : 0.f) + t2;
        if (dw1) dw1[(size_t)j * C + c] = (acc != 0.f ? acc * dw1[(size_t)j * C + c] : 0.f) + t1;
    }
    if (idx < C && db2) {
        float t = 0.f;
        for (int n = 0; n < N; ++n) t += dp2[(size_t)n * C + idx];
        db2[idx] = (acc != 0.f ? acc * db2[idx] : 0.f) + t;
    }
    if (idx < Cr && db1) {
        float t = 0.f;
        for (int n = 0; n < N; ++n) t += dp1[(size_t)n * Cr + idx];
        db1[idx] = (acc != 0.f ? acc * db1[idx] : 0.f) + t;
    }
}

__global__ void se_dgb_kernel(const float* __restrict__ sums2, int N, int C, float* dgamma, float* dbeta, float acc) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    double s = 0.0, q = 0.0;
    for (int n = 0; n < N; ++n) {
        s += (double)sums2[((size_t)n * C + c) * 2 + 0];
        q += (double)sums2[((size_t)n * C + c) * 2 + 1];
    }
    if (dbeta) dbeta[c] = (acc != 0.f ? acc * dbeta[c] : 0.f) + (float)s;
    if (dgamma) dgamma[c] = (acc != 0.f ? acc * dgamma[c] : 0.f) + (float)q;
}

// dz = gamma*rstd * (g - mean_v(g) - zhat * mean_v(g*zhat)),  g = mask * (dy*e + dm/V)
template <typename T, int VEC>
__global__ __launch_bounds__(256) void se_bwd_apply_kernel(const T* __restrict__ dy, int ldg, const T* __restrict__ z, int ldz,
                                                           T* __restrict__ dz, int ldo, int64_t V, int C, int Cr,
                                                           int cthreads, int rl, const float* __restrict__ stats,
                                                           const float* __restrict__ gamma, const float* __restrict__ beta,
                                                           const float* __restrict__ save, const float* __restrict__ dmv,
                                                           const float* __restrict__ sums2) {
    const int tid = threadIdx.x;
    const int cl = tid % cthreads, r0 = tid / cthreads;
    const int cv = blockIdx.z * 256 + cl;
    const int n = blockIdx.y;
    if (r0 >= rl || cv * VEC >= C) return;
    NormIn nm{stats, gamma, beta, C, 1};
    float a[VEC], b[VEC], mean[VEC], rstd[VEC], c1[VEC], c2[VEC], e[VEC], dm[VEC];
    const float invV = 1.0f / (float)V;
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        const size_t nc = (size_t)n * C + cv * VEC + i;
        norm_coeffs(nm, n, cv * VEC + i, a[i], b[i]);
        mean[i] = stats[nc * 2];
        rstd[i] = stats[nc * 2 + 1];
        c1[i] = sums2[nc * 2] * invV;
        c2[i] = sums2[nc * 2 + 1] * invV;
        e[i] = save[(size_t)n * (4 * C + Cr) + C + cv * VEC + i];
        dm[i] = dmv[nc];
    }
    const T* zb = z + ((int64_t)n * V) * ldz + (int64_t)cv * VEC;
    const T* gb = dy + ((int64_t)n * V) * ldg + (int64_t)cv * VEC;
    T* ob = dz + ((int64_t)n * V) * ldo + (int64_t)cv * VEC;
    for (int64_t r = (int64_t)blockIdx.x * rl + r0; r < V; r += (int64_t)gridDim.x * rl) {
        float v[VEC], g[VEC];
        Vec<T, VEC>::load(zb + r * ldz, v);
        Vec<T, VEC>::load(gb + r * ldg, g);
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            const float u = norm_u(v[i], a[i], b[i]);
            const float gg = u > 0.f ? fmaf(g[i], e[i], dm[i]) : 0.f;
            const float zh = (v[i] - mean[i]) * rstd[i];
            v[i] = a[i] * (gg - c1[i] - zh * c2[i]);
        }
        Vec<T, VEC>::store(ob + r * ldo, v);
    }
}

static int se_apply_blocks(int64_t V, int rl) {
    int64_t b = ((V + rl - 1) / rl + 3) / 4;
    if (b < 1) b = 1;
    return (int)(b > 4096 ? 4096 : b);
}

static lamp_status se_check(const lamp_tensor_desc* zd, int cr) {
    if (!desc_ok(zd)) return LAMP_ERR_SHAPE;
    if (cr < 1 || cr > 1024 || zd->c > 4096) return LAMP_ERR_SHAPE;
    return LAMP_OK;
}

// a[i] += b[i] in the storage dtype (fp32 sum, one rounding): the two gradients that meet at a shortcut.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void add_inplace_kernel(T* __restrict__ a, const T* __restrict__ b, int64_t nvec) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * 256) {
        float x[VEC], y[VEC];
        Vec<T, VEC>::load(a + i * VEC, x);
        Vec<T, VEC>::load(b + i * VEC, y);
#pragma unroll
        for (int k = 0; k < VEC; ++k) x[k] += y[k];
        Vec<T, VEC>::store(a + i * VEC, x);
    }
}

lamp_status launch_add_inplace(void* a, const void* b, int64_t numel, int dtype, hipStream_t s) {
    if (numel <= 0) return LAMP_OK;
    const int full = dtype == LAMP_BF16 ? 8 : 4;
    const int vec = (numel % full == 0 && aligned16(a) && aligned16(b)) ? full : 1;
    const int64_t nvec = numel / vec;
    const int64_t want = (nvec + 255) / 256;
    const int blocks = (int)(want < 256 * 32 ? want : 256 * 32);
    LAMP_DISPATCH_TV(dtype, vec, {
        hipLaunchKernelGGL((add_inplace_kernel<T, VEC>), dim3(blocks), dim3(256), 0, s, (T*)a, (const T*)b, nvec);
    });
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}

}  // namespace lamp

using namespace lamp;

extern "C" size_t lamp_inorm_relu_se_workspace_bytes(const lamp_tensor_desc* zd, int cr) {
    if (!zd || se_check(zd, cr) != LAMP_OK) return 0;
    const int64_t V = (int64_t)zd->d * zd->h * zd->w;
    const size_t nc = (size_t)zd->n * zd->c;
    return align_up(nc * stats_chunks(V) * 3 * sizeof(float)) + align_up(nc * 3 * sizeof(float)) +
           align_up(nc * 2 * sizeof(float)) + 2 * align_up(nc * sizeof(float)) +
           align_up((size_t)zd->n * cr * sizeof(float)) + 256;
}

extern "C" lamp_status lamp_inorm_relu_se(const lamp_tensor_desc* zd, const void* z, const float* stats, const float* gamma,
                                          const float* beta, int cr, const float* w1, const float* b1, const float* w2,
                                          const float* b2, const lamp_tensor_desc* rd, const void* residual,
                                          const lamp_tensor_desc* yd, void* y, float* gate_save, void* ws, size_t ws_bytes,
                                          void* stream) {
    if (!zd || !yd || !z || !y || !stats || !w1 || !w2 || !gate_save) return LAMP_ERR_NULL;
    lamp_status st = se_check(zd, cr);
    if (st != LAMP_OK) return st;
    if (!desc_ok(yd) || !same_space(zd, yd) || zd->c != yd->c) return LAMP_ERR_SHAPE;
    if (zd->dtype != yd->dtype) return LAMP_ERR_DTYPE;
    if (residual) {
        if (!rd) return LAMP_ERR_NULL;
        if (!desc_ok(rd) || !same_space(zd, rd) || rd->c != zd->c) return LAMP_ERR_SHAPE;
        if (rd->dtype != zd->dtype) return LAMP_ERR_DTYPE;
    }
    if (!ws || ws_bytes < lamp_inorm_relu_se_workspace_bytes(zd, cr)) return LAMP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int64_t V = (int64_t)zd->d * zd->h * zd->w;
    const int C = zd->c, chunks = stats_chunks(V);
    const int rpc = (int)((V + chunks - 1) / chunks);
    Carver cv(ws, ws_bytes);
    float* partial = (float*)cv.take((size_t)zd->n * C * chunks * 3 * sizeof(float));
    float* asum = (float*)cv.take((size_t)zd->n * C * 3 * sizeof(float));
    if (!cv.ok()) return LAMP_ERR_WORKSPACE;
    const int vec = pick_vec(zd->dtype, C, {zd->ldc, yd->ldc, residual ? rd->ldc : 0}, {z, y, residual});
    LAMP_DISPATCH_TV(zd->dtype, vec, {
        RowMap m = make_rowmap(C, VEC);
        hipLaunchKernelGGL((se_partial_kernel<T, VEC, 0>), dim3(chunks, zd->n, m.ctiles), dim3(256), 0, s, (const T*)nullptr, 0,
                           (const T*)z, zd->ldc, V, C, m.cthreads, m.rl, rpc, stats, gamma, beta, partial);
    });
    LAMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(se_finalize_kernel<3>, dim3(C, zd->n), dim3(256), 0, s, partial, chunks, C, asum);
    LAMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(se_gate_kernel, dim3(zd->n), dim3(256), (size_t)(C + cr) * sizeof(float), s, asum, 1.0f / (float)V, C, cr,
                       w1, b1, w2, b2, gate_save);
    LAMP_CHECK_LAUNCH();
    LAMP_DISPATCH_TV(zd->dtype, vec, {
        RowMap m = make_rowmap(C, VEC);
        const dim3 grid(se_apply_blocks(V, m.rl), zd->n, m.ctiles);
        if (residual)
            hipLaunchKernelGGL((se_apply_kernel<T, VEC, true>), grid, dim3(256), 0, s, (const T*)z, zd->ldc, (const T*)residual,
                               rd->ldc, (T*)y, yd->ldc, V, C, cr, m.cthreads, m.rl, stats, gamma, beta, gate_save);
        else
            hipLaunchKernelGGL((se_apply_kernel<T, VEC, false>), grid, dim3(256), 0, s, (const T*)z, zd->ldc, (const T*)nullptr,
                               0, (T*)y, yd->ldc, V, C, cr, m.cthreads, m.rl, stats, gamma, beta, gate_save);
    });
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}

extern "C" lamp_status lamp_inorm_relu_se_bwd(const lamp_tensor_desc* dyd, const void* dy, const lamp_tensor_desc* zd,
                                              const void* z, const float* stats, const float* gamma, const float* beta,
                                              int cr, const float* w1, const float* w2, const float* gate_save,
                                              const lamp_tensor_desc* dzd, void* dz, float* dgamma, float* dbeta, float* dw1,
                                              float* db1, float* dw2, float* db2, float beta_acc, void* ws, size_t ws_bytes,
                                              void* stream) {
    if (!dyd || !zd || !dzd || !dy || !z || !stats || !dz || !w1 || !w2 || !gate_save) return LAMP_ERR_NULL;
    lamp_status st = se_check(zd, cr);
    if (st != LAMP_OK) return st;
    if (!desc_ok(dyd) || !desc_ok(dzd) || !same_space(zd, dyd) || !same_space(zd, dzd) || zd->c != dyd->c || zd->c != dzd->c)
        return LAMP_ERR_SHAPE;
    if (zd->dtype != dyd->dtype || zd->dtype != dzd->dtype) return LAMP_ERR_DTYPE;
    if (beta_acc != 0.f && beta_acc != 1.f) return LAMP_ERR_SHAPE;
    if (!ws || ws_bytes < lamp_inorm_relu_se_workspace_bytes(zd, cr)) return LAMP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int64_t V = (int64_t)zd->d * zd->h * zd->w;
    const int C = zd->c, N = zd->n, chunks = stats_chunks(V);
    const int rpc = (int)((V + chunks - 1) / chunks);
    const size_t nc = (size_t)N * C;
    Carver cv(ws, ws_bytes);
    float* partial = (float*)cv.take(nc * chunks * 3 * sizeof(float));
    float* s3 = (float*)cv.take(nc * 3 * sizeof(float));
    float* sums2 = (float*)cv.take(nc * 2 * sizeof(float));
    float* dmv = (float*)cv.take(nc * sizeof(float));
    float* dp2 = (float*)cv.take(nc * sizeof(float));
    float* dp1 = (float*)cv.take((size_t)N * cr * sizeof(float));
    if (!cv.ok()) return LAMP_ERR_WORKSPACE;
    const int vec = pick_vec(zd->dtype, C, {zd->ldc, dyd->ldc, dzd->ldc}, {z, dy, dz});
    LAMP_DISPATCH_TV(zd->dtype, vec, {
        RowMap m = make_rowmap(C, VEC);
        hipLaunchKernelGGL((se_partial_kernel<T, VEC, 1>), dim3(chunks, N, m.ctiles), dim3(256), 0, s, (const T*)dy, dyd->ldc,
                           (const T*)z, zd->ldc, V, C, m.cthreads, m.rl, rpc, stats, gamma, beta, partial);
    });
    LAMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(se_finalize_kernel<3>, dim3(C, N), dim3(256), 0, s, partial, chunks, C, s3);
    LAMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(se_gate_bwd_kernel, dim3(N), dim3(256), (size_t)(C + cr) * sizeof(float), s, s3, 1.0f / (float)V, C, cr,
                       w1, w2, gate_save, dp2, dp1, dmv, sums2);
    LAMP_CHECK_LAUNCH();
    if (dw1 || db1 || dw2 || db2) {
        hipLaunchKernelGGL(se_param_grad_kernel, dim3(cdiv((int64_t)C * cr, 256)), dim3(256), 0, s, dp2, dp1, gate_save, N, C, cr,
                           dw1, db1, dw2, db2, beta_acc);
        LAMP_CHECK_LAUNCH();
    }
    if (dgamma || dbeta) {
        hipLaunchKernelGGL(se_dgb_kernel, dim3(cdiv(C, 64)), dim3(64), 0, s, sums2, N, C, dgamma, dbeta, beta_acc);
        LAMP_CHECK_LAUNCH();
    }
    LAMP_DISPATCH_TV(zd->dtype, vec, {
        RowMap m = make_rowmap(C, VEC);
        hipLaunchKernelGGL((se_bwd_apply_kernel<T, VEC>), dim3(se_apply_blocks(V, m.rl), N, m.ctiles), dim3(256), 0, s,
                           (const T*)dy, dyd->ldc, (const T*)z, zd->ldc, (T*)dz, dzd->ldc, V, C, cr, m.cthreads, m.rl, stats,
                           gamma, beta, gate_save, dmv, sums2);
    });
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}
