// RMSProp parameter update, every tensor of the network in one launch (bound by HBM: 22 bytes per
// parameter).
#include "internal.h"

namespace lamp {

struct RmsJob { float* w; float* v; const float* g; void* out; int64_t n; int out_bf16; int blk0; };
struct RmsBatch {
    int count;
    float lr, alpha, eps;
    RmsJob j[48];
};

// One thread per 4 consecutive parameters (scalar tail): v = alpha v + (1 - alpha) g^2,
// w -= lr g / (sqrt(v) + eps), working copy = w rounded to its storage type.
__global__ __launch_bounds__(256) void rmsprop_kernel(RmsBatch b) {
    int k = 0;
    while (k + 1 < b.count && (int)blockIdx.x >= b.j[k + 1].blk0) ++k;
    const RmsJob& q = b.j[k];
    const int64_t i0 = ((int64_t)((int)blockIdx.x - q.blk0) * 256 + threadIdx.x) * 4;
    if (i0 >= q.n) return;
    const int cnt = q.n - i0 >= 4 ? 4 : (int)(q.n - i0);
    float w[4], v[4], g[4];
    const bool vec = cnt == 4 && ((((uintptr_t)(q.w + i0)) | ((uintptr_t)(q.v + i0)) | ((uintptr_t)(q.g + i0))) & 15u) == 0;
    if (vec) {
        const float4 w4 = *reinterpret_cast<const float4*>(q.w + i0), v4 = *reinterpret_cast<const float4*>(q.v + i0),
                     g4 = *reinterpret_cast<const float4*>(q.g + i0);
        w[0] = w4.x; w[1] = w4.y; w[2] = w4.z; w[3] = w4.w;
        v[0] = v4.x; v[1] = v4.y; v[2] = v4.z; v[3] = v4.w;
        g[0] = g4.x; g[1] = g4.y; g[2] = g4.z; g[3] = g4.w;
    } else {
        for (int e = 0; e < cnt; ++e) { w[e] = q.w[i0 + e]; v[e] = q.v[i0 + e]; g[e] = q.g[i0 + e]; }
    }
    for (int e = 0; e < cnt; ++e) {
        v[e] = b.alpha * v[e] + (1.f - b.alpha) * g[e] * g[e];
        w[e] = w[e] - b.lr * g[e] / (sqrtf(v[e]) + b.eps);
    }
    if (vec) {
        *reinterpret_cast<float4*>(q.w + i0) = make_float4(w[0], w[1], w[2], w[3]);
        *reinterpret_cast<float4*>(q.v + i0) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
        for (int e = 0; e < cnt; ++e) { q.w[i0 + e] = w[e]; q.v[i0 + e] = v[e]; }
    }
    if (q.out) {
        if (q.out_bf16) {
            bf16_t* o = (bf16_t*)q.out + i0;
            for (int e = 0; e < cnt; ++e) o[e] = f2bf(w[e]);
        } else if (q.out != (void*)q.w) {
            float* o = (float*)q.out + i0;
            for (int e = 0; e < cnt; ++e) o[e] = w[e];
        }
    }
}

}  // namespace lamp

using namespace lamp;

extern "C" lamp_status lamp_rmsprop_step(int32_t count, const int64_t* numel, float* const* w, float* const* v,
                                         const float* const* g, void* const* w_out, const int32_t* out_dtype, float lr,
                                         float alpha, float eps, void* stream) {
    if (count < 0) return LAMP_ERR_SHAPE;
    if (count == 0) return LAMP_OK;
    if (!numel || !w || !v || !g) return LAMP_ERR_NULL;
    if (!(lr >= 0.f) || !(alpha >= 0.f && alpha <= 1.f) || !(eps >= 0.f)) return LAMP_ERR_SHAPE;
    for (int i = 0; i < count; ++i) {
        if (numel[i] < 0) return LAMP_ERR_SHAPE;
        if (numel[i] > 0 && (!w[i] || !v[i] || !g[i])) return LAMP_ERR_NULL;
        if (w_out && w_out[i]) {
            if (!out_dtype) return LAMP_ERR_NULL;
            if (out_dtype[i] != LAMP_F32 && out_dtype[i] != LAMP_BF16) return LAMP_ERR_DTYPE;
        }
    }
    hipStream_t s = (hipStream_t)stream;
    for (int first = 0; first < count; first += 48) {
        RmsBatch b;
        b.lr = lr; b.alpha = alpha; b.eps = eps;
        b.count = 0;
        int64_t blk = 0;
        for (int i = first; i < count && i < first + 48; ++i) {
            if (numel[i] == 0) continue;
            RmsJob& q = b.j[b.count++];
            q.w = w[i]; q.v = v[i]; q.g = g[i]; q.n = numel[i];
            q.out = w_out ? w_out[i] : nullptr;
            q.out_bf16 = (q.out && out_dtype[i] == LAMP_BF16) ? 1 : 0;
            q.blk0 = (int)blk;
            blk += cdiv(cdiv(numel[i], 4), 256);
            if (blk >= ((int64_t)1 << 31)) return LAMP_ERR_SHAPE;
        }
        if (b.count == 0) continue;
        hipLaunchKernelGGL(rmsprop_kernel, dim3((unsigned)blk), dim3(256), 0, s, b);
        LAMP_CHECK_LAUNCH();
    }
    return LAMP_OK;
}
