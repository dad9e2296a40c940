// Internal helpers shared by the HIP translation units of liblamp (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/lamp.h"

namespace lamp {

typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
// round-to-nearest-even; NaN/Inf are out of contract
__device__ __forceinline__ bf16_t f2bf(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename T> struct io;
template <> struct io<float> {
    static __device__ __forceinline__ float ld(const float* p) { return *p; }
    static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
    static __device__ __forceinline__ float rnd(float v) { return v; }
};
template <> struct io<bf16_t> {
    static __device__ __forceinline__ float ld(const bf16_t* p) { return bf2f(*p); }
    static __device__ __forceinline__ void st(bf16_t* p, float v) { *p = f2bf(v); }
    static __device__ __forceinline__ float rnd(float v) { return bf2f(f2bf(v)); }
};

// Device-side view of lamp_norm_in plus the batch stride of its statistics.
struct NormIn {
    const float* mean_rstd;  // [N][c_norm][2] or nullptr (= no transform)
    const float* gamma;
    const float* beta;
    int c_norm;
    int relu;
};

// The one formula for the normalised pre-activation used by every kernel (forward apply,
// normalise-on-load and the ReLU mask of the backward), so masks agree bit for bit.
__device__ __forceinline__ void norm_coeffs(const NormIn& nm, int n, int c, float& a, float& b) {
    float mean = nm.mean_rstd[((size_t)n * nm.c_norm + c) * 2 + 0];
    float rstd = nm.mean_rstd[((size_t)n * nm.c_norm + c) * 2 + 1];
    float g = nm.gamma ? nm.gamma[c] : 1.0f;
    float bt = nm.beta ? nm.beta[c] : 0.0f;
    a = g * rstd;
    b = bt - mean * a;
}
__device__ __forceinline__ float norm_u(float z, float a, float b) { return fmaf(z, a, b); }

template <typename T>
__device__ __forceinline__ float load_norm(const T* p, const NormIn& nm, int n, int c) {
    float v = io<T>::ld(p);
    if (nm.mean_rstd && c < nm.c_norm) {
        float a, b;
        norm_coeffs(nm, n, c, a, b);
        v = norm_u(v, a, b);
        if (nm.relu) v = v > 0.0f ? v : 0.0f;
        v = io<T>::rnd(v);  // the activated tensor is a storage-dtype tensor
    }
    return v;
}

inline NormIn make_norm(const lamp_norm_in* p) {
    NormIn n;
    if (p && p->mean_rstd && p->c_norm > 0) {
        n.mean_rstd = p->mean_rstd; n.gamma = p->gamma; n.beta = p->beta; n.c_norm = p->c_norm; n.relu = p->relu;
    } else {
        n.mean_rstd = nullptr; n.gamma = nullptr; n.beta = nullptr; n.c_norm = 0; n.relu = 0;
    }
    return n;
}

// ---- host-side validation helpers ---------------------------------------------------------
inline bool desc_ok(const lamp_tensor_desc* t) {
    return t && t->n > 0 && t->d > 0 && t->h > 0 && t->w > 0 && t->c > 0 && t->ldc >= t->c &&
           (t->dtype == LAMP_F32 || t->dtype == LAMP_BF16);
}
inline bool same_space(const lamp_tensor_desc* a, const lamp_tensor_desc* b) {
    return a->n == b->n && a->d == b->d && a->h == b->h && a->w == b->w;
}
inline size_t esize(int dtype) { return dtype == LAMP_BF16 ? 2 : 4; }
inline int64_t nvox(const lamp_tensor_desc* t) { return (int64_t)t->n * t->d * t->h * t->w; }
inline bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }
inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }
inline lamp_status norm_ok(const lamp_norm_in* nm, const lamp_tensor_desc* xd) {
    if (!nm || !nm->mean_rstd) return LAMP_OK;
    if (nm->c_norm < 0 || nm->c_norm > xd->c) return LAMP_ERR_SHAPE;
    return LAMP_OK;
}

#define LAMP_CHECK_LAUNCH()                                   \
    do {                                                      \
        if (hipGetLastError() != hipSuccess) return LAMP_ERR_HIP; \
    } while (0)

// Simple bump allocator over the caller's workspace.
struct Carver {
    char* base; size_t size; size_t off;
    Carver(void* p, size_t n) : base((char*)p), size(n), off(0) {}
    void* take(size_t bytes) {
        size_t o = align_up(off);
        if (!base || o + bytes > size) { off = size + 1; return nullptr; }
        off = o + bytes;
        return base + o;
    }
    bool ok() const { return off <= size; }
};

static inline int cdiv(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

}  // namespace lamp
