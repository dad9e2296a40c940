// Deterministic second-stage reductions shared by the weight-gradient paths.
#include <mutex>
#include "internal.h"
#include "vec.h"

namespace lamp {

// 16 zero bytes in device memory: the source of the zero padding for the register-free global -> LDS
// copies.  A statically initialised device array that no kernel writes; `used` keeps it in the device
// code object although no kernel names it (a const array would have internal linkage and be dropped
// there, and the lookup below would then fail).  Its address is looked up once per device and checked
// (device memory, reads back as zeros) before any kernel gets it.
__device__ __attribute__((used, aligned(16))) uint32_t lamp_zero16_storage[4] = {0u, 0u, 0u, 0u};
const bf16_t* device_zero16() {
    static const bf16_t* cache[64] = {nullptr};
    static std::mutex mu;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (!cache[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(lamp_zero16_storage)) != hipSuccess || !p) return nullptr;
        hipPointerAttribute_t at;
        if (hipPointerGetAttributes(&at, p) != hipSuccess || at.type != hipMemoryTypeDevice) return nullptr;
        uint32_t back[4] = {1u, 1u, 1u, 1u};
        if (hipMemcpy(back, p, sizeof(back), hipMemcpyDeviceToHost) != hipSuccess) return nullptr;
        if (back[0] | back[1] | back[2] | back[3]) return nullptr;
        cache[dev] = (const bf16_t*)p;
    }
    return cache[dev];
}

// Block = (256/SL) outputs x SL lanes over the parts; every lane adds its strided parts in order,
// then the lanes are added in order: a fixed summation tree, fp64.
template <int SL>
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ part, int S, int64_t O,
                                                              float* __restrict__ out, float beta) {
    constexpr int OPB = 256 / SL;
    __shared__ double sh[SL][OPB];
    const int ol = threadIdx.x % OPB, sl = threadIdx.x / OPB;
    const int64_t o = (int64_t)blockIdx.x * OPB + ol;
    double acc = 0.0;
    if (o < O) {
        // eight loads in flight, added in the order of the parts: a loop of load-then-add is a chain of memory
        // latencies (32 of them for 256 parts), which is what this kernel's time was
        int s = sl;
        for (; s + 7 * SL < S; s += 8 * SL) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = part[(int64_t)(s + u * SL) * O + o];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += (double)v[u];
        }
        for (; s < S; s += SL) acc += (double)part[(int64_t)s * O + o];
    }
    sh[sl][ol] = acc;
    __syncthreads();
    if (sl == 0 && o < O) {
        double t = 0.0;
#pragma unroll
        for (int k = 0; k < SL; ++k) t += sh[k][ol];
        out[o] = (beta != 0.f ? beta * out[o] : 0.f) + (float)t;
    }
}

lamp_status launch_reduce_partials(const float* part, int S, int64_t O, float* out, float beta, hipStream_t s) {
    if (O <= 16384 && S >= 64)
        hipLaunchKernelGGL((reduce_partials_kernel<64>), dim3(cdiv(O, 4)), dim3(256), 0, s, part, S, O, out, beta);
    else if (S >= 8)
        hipLaunchKernelGGL((reduce_partials_kernel<8>), dim3(cdiv(O, 32)), dim3(256), 0, s, part, S, O, out, beta);
    else
        hipLaunchKernelGGL((reduce_partials_kernel<1>), dim3(cdiv(O, 256)), dim3(256), 0, s, part, S, O, out, beta);
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}

// rows per chunk: about 2048 chunks, at least 32 rows each
static int col_rows(int64_t rows) {
    int64_t r = (rows + 2047) / 2048;
    return (int)(r < 32 ? 32 : r);
}

// Threads side by side cover the channel vectors of one row; the row lanes are added in order.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void colsum_partial_kernel(const T* __restrict__ t, int64_t rows, int C, int ld,
                                                             int rows_per_chunk, float* __restrict__ part, RowMap m) {
    __shared__ float red[VEC][256];
    const int tid = threadIdx.x, cl = tid % m.cthreads, r0 = tid / m.cthreads;
    const int c0 = (blockIdx.y * 256 + cl) * VEC;
    int64_t rbeg = (int64_t)blockIdx.x * rows_per_chunk, rend = rbeg + rows_per_chunk;
    if (rend > rows) rend = rows;
    float s[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) s[i] = 0.f;
    if (r0 < m.rl && c0 < C)
        for (int64_t r = rbeg + r0; r < rend; r += m.rl) {
            float v[VEC];
            Vec<T, VEC>::load(t + r * ld + c0, v);
#pragma unroll
            for (int i = 0; i < VEC; ++i) s[i] += v[i];
        }
#pragma unroll
    for (int i = 0; i < VEC; ++i) red[i][tid] = s[i];
    __syncthreads();
    if (r0 == 0 && c0 < C) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            float ss = 0.f;
            for (int r = 0; r < m.rl; ++r) ss += red[i][r * m.cthreads + cl];
            part[(int64_t)blockIdx.x * C + c0 + i] = ss;
        }
    }
}

size_t colsum_ws_bytes(int64_t rows, int C) {
    const int cr = col_rows(rows);
    int64_t chunks = (rows + cr - 1) / cr;
    return align_up((size_t)chunks * C * sizeof(float));
}

lamp_status launch_colsum(const void* t, int dtype, int64_t rows, int C, int ld, float* out, float beta, void* ws,
                          size_t ws_bytes, hipStream_t s) {
    const int cr = col_rows(rows);
    int chunks = (int)((rows + cr - 1) / cr);
    if (!ws || ws_bytes < colsum_ws_bytes(rows, C)) return LAMP_ERR_WORKSPACE;
    float* part = (float*)ws;
    const int vec = pick_vec(dtype, C, {ld}, {t});
    const RowMap m = make_rowmap(C, vec);
    dim3 grid(chunks, m.ctiles);
    LAMP_DISPATCH_TV(dtype, vec, {
        hipLaunchKernelGGL((colsum_partial_kernel<T, VEC>), grid, dim3(256), 0, s, (const T*)t, rows, C, ld, cr, part, m);
    });
    LAMP_CHECK_LAUNCH();
    return launch_reduce_partials(part, chunks, C, out, beta, s);
}

}  // namespace lamp
