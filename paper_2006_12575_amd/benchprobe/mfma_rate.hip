// Bench-only helper, not part of liblamp: the rate at which this GPU executes a register-resident loop of
// the bf16 32x32x16 matrix-core instruction the convolution kernels use (no memory or LDS traffic), one
// wave per SIMD.  The rate depends on the operand values (switching power sets the clock), which bounds
// what any kernel reaches on real activations; bench.py prints it beside the published peak.
// This helper allocates and frees a small device buffer and synchronises, which is why it lives in a
// library of its own (liblamp_benchprobe.so) and not behind the product's ABI.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

__global__ __launch_bounds__(256) void mfma_rate_kernel(const uint4* __restrict__ src, float* __restrict__ out, int iters,
                                                        int nfrag) {
    extern __shared__ __attribute__((aligned(16))) char lds[];   // sized so that one workgroup fits per CU
    f32x16 acc[8];
    for (int i = 0; i < 8; ++i)
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    bf16x8 a[4], b[4];
    for (int i = 0; i < 4; ++i) {
        a[i] = __builtin_bit_cast(bf16x8, src[(threadIdx.x * 8 + i) % nfrag]);
        b[i] = __builtin_bit_cast(bf16x8, src[(threadIdx.x * 8 + 4 + i) % nfrag]);
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < 24; ++m)
            acc[m & 7] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m & 3], b[(m >> 2) & 3], acc[m & 7], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 8; ++i)
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__device__ __forceinline__ uint16_t to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__global__ void fill_kernel(uint32_t* __restrict__ p, int n, int pattern) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint32_t v = 0u;
    if (pattern == 1) {
        // two bf16 values ~ N(0,1): sum of 12 uniforms from a counter-based integer hash, minus 6
        float f[2];
        for (int h = 0; h < 2; ++h) {
            float u = 0.f;
            for (int j = 0; j < 12; ++j) {
                uint32_t x = (uint32_t)(i * 2 + h) * 12u + (uint32_t)j + 0x9E3779B9u;
                x ^= x >> 16; x *= 0x7FEB352Du; x ^= x >> 15; x *= 0x846CA68Bu; x ^= x >> 16;
                u += (float)(x >> 8) * (1.0f / 16777216.0f);
            }
            f[h] = u - 6.f;
        }
        v = (uint32_t)to_bf16(f[0]) | ((uint32_t)to_bf16(f[1]) << 16);
    }
    p[i] = v;
}
}  // namespace

// pattern 0 = zero operands, 1 = standard-normal operands (seeded).  Writes TFLOP/s to *tflops.
// Returns 0 on success, -1 on a bad argument, -2 on a HIP error.  Runs on the default stream and waits.
extern "C" int benchprobe_mfma_rate(int32_t pattern, int32_t iters, float* tflops) {
    if (!tflops || pattern < 0 || pattern > 1 || iters < 1) return -1;
    const int nfrag = 4096, blocks = 256, shm = 100 * 1024;
    char* buf = nullptr;
    if (hipMalloc(&buf, (size_t)nfrag * 16 + (size_t)blocks * 256 * sizeof(float)) != hipSuccess) return -2;
    uint4* src = (uint4*)buf;
    float* out = (float*)(buf + (size_t)nfrag * 16);
    int rc = 0;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    do {
        if (hipFuncSetAttribute((const void*)mfma_rate_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, shm) != hipSuccess ||
            hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) { rc = -2; break; }
        hipLaunchKernelGGL(fill_kernel, dim3(nfrag * 4 / 256), dim3(256), 0, 0, (uint32_t*)src, nfrag * 4, pattern);
        hipLaunchKernelGGL(mfma_rate_kernel, dim3(blocks), dim3(256), shm, 0, src, out, 64, nfrag);   // warm-up
        if (hipEventRecord(e0, 0) != hipSuccess) { rc = -2; break; }
        hipLaunchKernelGGL(mfma_rate_kernel, dim3(blocks), dim3(256), shm, 0, src, out, iters, nfrag);
        if (hipEventRecord(e1, 0) != hipSuccess || hipEventSynchronize(e1) != hipSuccess || hipGetLastError() != hipSuccess) {
            rc = -2;
            break;
        }
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess || ms <= 0.f) { rc = -2; break; }
        *tflops = (float)((double)blocks * 4 * iters * 24 * 32768.0 / ms / 1e9);
    } while (0);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(buf);
    return rc;
}
