// Status strings and build information.
#include "common.h"

extern "C" const char* lamp_status_string(lamp_status s) {
    switch (s) {
        case LAMP_OK: return "ok";
        case LAMP_ERR_NULL: return "a required pointer is NULL";
        case LAMP_ERR_SHAPE: return "bad or mismatching shape";
        case LAMP_ERR_ALIGN: return "pointer or stride not aligned";
        case LAMP_ERR_DTYPE: return "unknown or mismatching dtype";
        case LAMP_ERR_WORKSPACE: return "workspace missing or too small";
        case LAMP_ERR_UNSUPPORTED: return "unsupported request";
        case LAMP_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

extern "C" const char* lamp_build_info(void) { return "liblamp 0.1 gfx950"; }

// ---- diagnostic: matrix-core rate of a register-resident loop as a function of the operand values
namespace lamp {
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 probe_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float probe_f32x16;
__global__ __launch_bounds__(256) void mfma_rate_kernel(const uint4* __restrict__ src, float* __restrict__ out, int iters,
                                                        int nfrag) {
    extern __shared__ __attribute__((aligned(16))) char lds[];   // sized so that one workgroup fits per CU
    probe_f32x16 acc[8];
    for (int i = 0; i < 8; ++i)
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    probe_bf16x8 a[4], b[4];
    for (int i = 0; i < 4; ++i) {
        a[i] = __builtin_bit_cast(probe_bf16x8, src[(threadIdx.x * 8 + i) % nfrag]);
        b[i] = __builtin_bit_cast(probe_bf16x8, src[(threadIdx.x * 8 + 4 + i) % nfrag]);
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
// The same loop at the conv kernel's design point: operands fresh from LDS (12 fragment reads of 16 bytes
// per lane and 24 MFMAs, double buffered in registers), the kernel's filler ratio beside them (62 VALU and
// 45 SALU instructions per 24 MFMAs, measured on conv3d_ring_kernel) and 3 register-free global -> LDS
// copies per 24 MFMAs from a cache-resident buffer.  No barriers, no dependence on memory latency: what
// perfect scheduling of that instruction mix would reach on this data.
__global__ __launch_bounds__(256) void mfma_mix_kernel(const uint4* __restrict__ src, float* __restrict__ out, int iters,
                                                       int nfrag) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    for (int i = tid; i < 4096; i += 256) reinterpret_cast<uint4*>(lds)[i] = src[i % nfrag];   // 64 KB of operand data
    __syncthreads();
    probe_f32x16 acc[8];
    for (int i = 0; i < 8; ++i)
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    const char* base = lds + wv * 16384 + lane * 16;   // this wave's 16 KB; fragment f at base + 1024 * f
    probe_bf16x8 fa[12], fb[12];
    for (int f = 0; f < 12; ++f) {
        fa[f] = __builtin_bit_cast(probe_bf16x8, *reinterpret_cast<const uint4*>(base + f * 1024));
        fb[f] = fa[f];
    }
    float x0 = (float)tid, x1 = 1.f, y = 0.5f;
    int s0 = iters;
    char* dma = lds + 65536 + wv * 1024;
    // one pass: 24 MFMAs on `use`, the 12 fragments of the next pass read into `fill` meanwhile
    auto pass = [&](const probe_bf16x8 (&use)[12], probe_bf16x8 (&fill)[12], int rot, int it) __attribute__((always_inline)) {
#pragma unroll
        for (int m = 0; m < 24; ++m) {
            acc[m & 7] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(use[m % 6], use[6 + (m / 4) % 6], acc[m & 7], 0, 0, 0);
            if ((m & 1) == 0)
                fill[m >> 1] = __builtin_bit_cast(probe_bf16x8, *reinterpret_cast<const uint4*>(base + ((rot + (m >> 1)) & 15) * 1024));
#pragma unroll
            for (int f = 0; f < (62 * (m + 1)) / 24 - (62 * m) / 24; ++f) {
                if (f & 1) asm volatile("v_add_f32 %0, %0, %1" : "+v"(x1) : "v"(y));
                else asm volatile("v_add_f32 %0, %0, %1" : "+v"(x0) : "v"(y));
            }
#pragma unroll
            for (int f = 0; f < (45 * (m + 1)) / 24 - (45 * m) / 24; ++f) asm volatile("s_add_u32 %0, %0, 1" : "+s"(s0));
            if (m % 8 == 0) {
                const uint32_t m0v = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)dma);
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                             ::"s"(m0v), "v"(src + (((it * 3 + m) & 63) * 64 + lane) % nfrag) : "memory", "m0");
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
    };
    for (int it = 0; it < iters; it += 4) {   // iters is rounded up to a multiple of 4 by the host
        pass(fa, fb, 0, it);
        pass(fb, fa, 12, it + 1);
        pass(fa, fb, 8, it + 2);
        pass(fb, fa, 4, it + 3);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    float s = x0 + x1 + (float)s0;
    for (int i = 0; i < 8; ++i)
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}
__global__ void mfma_rate_fill_kernel(uint32_t* __restrict__ p, int n, int pattern) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint32_t v = 0u;
    if (pattern >= 1) {
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
        v = (uint32_t)f2bf(f[0]) | ((uint32_t)f2bf(f[1]) << 16);
    }
    p[i] = v;
}
}  // namespace lamp

extern "C" lamp_status lamp_probe_mfma_rate(int32_t pattern, int32_t iters, float* tflops, void* stream) {
    using namespace lamp;
    if (!tflops) return LAMP_ERR_NULL;
    if (pattern < 0 || pattern > 2 || iters < 1) return LAMP_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    const int nfrag = 4096, blocks = 256, shm = 100 * 1024;
    char* buf = nullptr;
    if (hipMalloc(&buf, (size_t)nfrag * 16 + (size_t)blocks * 256 * sizeof(float)) != hipSuccess) return LAMP_ERR_HIP;
    uint4* src = (uint4*)buf;
    float* out = (float*)(buf + (size_t)nfrag * 16);
    lamp_status st = LAMP_OK;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    do {
        void (*kern)(const uint4*, float*, int, int) = pattern == 2 ? mfma_mix_kernel : mfma_rate_kernel;
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, shm) != hipSuccess ||
            hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) { st = LAMP_ERR_HIP; break; }
        hipLaunchKernelGGL(mfma_rate_fill_kernel, dim3(nfrag * 4 / 256), dim3(256), 0, s, (uint32_t*)src, nfrag * 4, pattern);
        hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), shm, s, src, out, 64, nfrag);   // warm-up
        if (hipEventRecord(e0, s) != hipSuccess) { st = LAMP_ERR_HIP; break; }
        iters = (iters + 3) & ~3;   // the mixed loop is unrolled four times
        hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), shm, s, src, out, iters, nfrag);
        if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess || hipGetLastError() != hipSuccess) {
            st = LAMP_ERR_HIP;
            break;
        }
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess || ms <= 0.f) { st = LAMP_ERR_HIP; break; }
        *tflops = (float)((double)blocks * 4 * iters * 24 * 32768.0 / ms / 1e9);
    } while (0);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(buf);
    return st;
}
