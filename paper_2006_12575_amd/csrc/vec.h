// Vector load/store helpers and the (channel-vector, row-lane) thread mapping used by the
// bandwidth-bound NDHWC kernels.
#pragma once
#include <initializer_list>
#include "common.h"

namespace lamp {

template <typename T, int VEC> struct Vec;

template <> struct Vec<bf16_t, 8> {
    static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[8]) {
        uint4 q = *reinterpret_cast<const uint4*>(p);
        uint32_t r[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(r[i] << 16);
            v[2 * i + 1] = __uint_as_float(r[i] & 0xFFFF0000u);
        }
    }
    static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[8]) {
        uint32_t r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = (uint32_t)f2bf(v[2 * i]) | ((uint32_t)f2bf(v[2 * i + 1]) << 16);
        *reinterpret_cast<uint4*>(p) = make_uint4(r[0], r[1], r[2], r[3]);
    }
};
template <> struct Vec<float, 4> {
    static __device__ __forceinline__ void load(const float* p, float (&v)[4]) {
        float4 q = *reinterpret_cast<const float4*>(p);
        v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    }
    static __device__ __forceinline__ void store(float* p, const float (&v)[4]) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    }
};
template <typename T> struct Vec<T, 1> {
    static __device__ __forceinline__ void load(const T* p, float (&v)[1]) { v[0] = io<T>::ld(p); }
    static __device__ __forceinline__ void store(T* p, const float (&v)[1]) { io<T>::st(p, v[0]); }
};

// Thread mapping inside a 256-thread block: cthreads threads side by side cover the channel
// vectors of one row, rl rows are in flight per block.  Channel-vector tiles beyond 256 go to
// blockIdx.z.
struct RowMap {
    int cthreads, rl, ctiles;
};
inline RowMap make_rowmap(int C, int VEC) {
    RowMap m;
    int cv = C / VEC;
    m.cthreads = cv < 256 ? cv : 256;
    m.rl = 256 / m.cthreads;
    m.ctiles = (cv + 255) / 256;
    return m;
}
// Vector width usable for a tensor set: all channel counts / strides divisible and pointers aligned.
inline int pick_vec(int dtype, int C, std::initializer_list<int> lds, std::initializer_list<const void*> ptrs) {
    int v = dtype == LAMP_BF16 ? 8 : 4;
    if (C % v) return 1;
    for (int l : lds) if (l % v) return 1;
    for (const void* p : ptrs) if (p && (((uintptr_t)p) & 15u)) return 1;
    return v;
}

// Vector load with the optional normalise+ReLU-on-load transform.
template <typename T, int VEC>
__device__ __forceinline__ void load_norm_vec(const T* p, const NormIn& nm, int n, int c0, float (&v)[VEC]) {
    Vec<T, VEC>::load(p, v);
    if (nm.mean_rstd) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            int c = c0 + i;
            if (c < nm.c_norm) {
                float a, b;
                norm_coeffs(nm, n, c, a, b);
                float u = norm_u(v[i], a, b);
                if (nm.relu) u = u > 0.f ? u : 0.f;
                v[i] = io<T>::rnd(u);
            }
        }
    }
}

}  // namespace lamp

// Expands BODY with T / VEC bound to the storage type and vector width.
#define LAMP_DISPATCH_TV(dtype, vec, BODY)                                          \
    do {                                                                            \
        if ((dtype) == LAMP_BF16) {                                                 \
            if ((vec) == 8) { typedef bf16_t T; constexpr int VEC = 8; BODY }        \
            else { typedef bf16_t T; constexpr int VEC = 1; BODY }                   \
        } else {                                                                    \
            if ((vec) == 4) { typedef float T; constexpr int VEC = 4; BODY }         \
            else { typedef float T; constexpr int VEC = 1; BODY }                    \
        }                                                                           \
    } while (0)
