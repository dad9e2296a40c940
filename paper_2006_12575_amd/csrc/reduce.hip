// Deterministic second-stage reductions shared by the weight-gradient paths.
#include "internal.h"

namespace lamp {

__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ part, int S, int64_t O,
                                                              float* __restrict__ out, float beta) {
    int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (o >= O) return;
    double acc = 0.0;
    for (int s = 0; s < S; ++s) acc += (double)part[(int64_t)s * O + o];
    out[o] = (beta != 0.f ? beta * out[o] : 0.f) + (float)acc;
}

lamp_status launch_reduce_partials(const float* part, int S, int64_t O, float* out, float beta, hipStream_t s) {
    hipLaunchKernelGGL(reduce_partials_kernel, dim3(cdiv(O, 256)), dim3(256), 0, s, part, S, O, out, beta);
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}

static const int kColRows = 4096;

template <typename T>
__global__ __launch_bounds__(256) void colsum_partial_kernel(const T* __restrict__ t, int64_t rows, int C, int ld,
                                                             int rows_per_chunk, float* __restrict__ part) {
    __shared__ float red[256];
    const int cthreads = C < 256 ? C : 256;
    const int rl = 256 / cthreads;
    const int tid = threadIdx.x, cl = tid % cthreads, r0 = tid / cthreads;
    const int c = blockIdx.y * 256 + cl;
    int64_t rbeg = (int64_t)blockIdx.x * rows_per_chunk, rend = rbeg + rows_per_chunk;
    if (rend > rows) rend = rows;
    float s = 0.f;
    if (r0 < rl && c < C)
        for (int64_t r = rbeg + r0; r < rend; r += rl) s += io<T>::ld(t + r * ld + c);
    red[tid] = s;
    __syncthreads();
    if (r0 == 0 && c < C) {
        float ss = 0.f;
        for (int r = 0; r < rl; ++r) ss += red[r * cthreads + cl];
        part[(int64_t)blockIdx.x * C + c] = ss;
    }
}

size_t colsum_ws_bytes(int64_t rows, int C) {
    int64_t chunks = (rows + kColRows - 1) / kColRows;
    return align_up((size_t)chunks * C * sizeof(float));
}

lamp_status launch_colsum(const void* t, int dtype, int64_t rows, int C, int ld, float* out, float beta, void* ws,
                          size_t ws_bytes, hipStream_t s) {
    int chunks = (int)((rows + kColRows - 1) / kColRows);
    if (!ws || ws_bytes < colsum_ws_bytes(rows, C)) return LAMP_ERR_WORKSPACE;
    float* part = (float*)ws;
    dim3 grid(chunks, cdiv(C, 256));
    if (dtype == LAMP_BF16)
        hipLaunchKernelGGL((colsum_partial_kernel<bf16_t>), grid, dim3(256), 0, s, (const bf16_t*)t, rows, C, ld,
                           kColRows, part);
    else
        hipLaunchKernelGGL((colsum_partial_kernel<float>), grid, dim3(256), 0, s, (const float*)t, rows, C, ld, kColRows,
                           part);
    LAMP_CHECK_LAUNCH();
    return launch_reduce_partials(part, chunks, C, out, beta, s);
}

}  // namespace lamp
