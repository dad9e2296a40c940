// InstanceNorm + ReLU: statistics (two-stage, deterministic), apply, and backward.
// Bandwidth-bound kernels on NDHWC tensors; fp32 arithmetic, fp64 merging of partial moments.
#include <initializer_list>
#include <mutex>
#include "internal.h"
#include "vec.h"

// Scratch of the allocation-free entry point (lamp_inorm_relu_noalloc): partial moments and per-chunk counts of
// the statistics pass (LAMP_NOALLOC_SCRATCH_BYTES of the public header).  One copy per GPU, held until the process
// ends; every call on a GPU shares it.
static __device__ __align__(256) unsigned char scratch[LAMP_NOALLOC_SCRATCH_BYTES];

namespace lamp {

// Device address of `scratch` on the current device.  In host code the array's name is only a stand-in for
// the symbol, never an address a kernel may get: the address is looked up once per device, with that device
// current, and kept.
static lamp_status noalloc_scratch(void** out) {
    static std::mutex mu;
    static void* cache[64] = {nullptr};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return LAMP_ERR_HIP;
    std::lock_guard<std::mutex> lock(mu);
    if (!cache[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LAMP_ERR_HIP;
        cache[dev] = p;
    }
    *out = cache[dev];
    return LAMP_OK;
}


// Rows of one partial sum: about 2048 chunks per sample so that small volumes still fill the chip,
// never fewer than 32 rows.
static int rows_per_chunk(int64_t v) {
    const int64_t r = (v + 2047) / 2048;
    return (int)(r < 32 ? 32 : r);
}

int stats_chunks(int64_t v) {
    const int r = rows_per_chunk(v);
    return (int)((v + r - 1) / r);
}

size_t stats_ws_bytes(const lamp_tensor_desc* zd) {
    int64_t V = (int64_t)zd->d * zd->h * zd->w;
    int ch = stats_chunks(V);
    return align_up((size_t)zd->n * ch * zd->c * 2 * sizeof(float)) + align_up((size_t)ch * sizeof(int32_t));
}

// ---- forward statistics ---------------------------------------------------------------------
// partial[((n*chunks + chunk)*C + c)*2] = (sum, sum of squares) over the chunk's rows.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void stats_partial_kernel(const T* __restrict__ z, int ld, int64_t V, int C,
                                                            int cthreads, int rl, int rows_per_chunk,
                                                            float* __restrict__ partial, int32_t* __restrict__ counts) {
    __shared__ float red[2][256 * VEC];
    const int tid = threadIdx.x;
    const int cl = tid % cthreads, r0 = tid / cthreads;
    const int cv = blockIdx.z * 256 + cl;
    const int chunk = blockIdx.x, n = blockIdx.y, chunks = gridDim.x;
    const int64_t rbeg = (int64_t)chunk * rows_per_chunk;
    int64_t rend = rbeg + rows_per_chunk;
    if (rend > V) rend = V;
    float s[VEC], q[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) { s[i] = 0.f; q[i] = 0.f; }
    const bool active = r0 < rl && cv * VEC < C;
    if (active) {
        const T* base = z + ((int64_t)n * V) * ld + (int64_t)cv * VEC;
        int64_t r = rbeg + r0;
        // four rows in flight; the additions keep the row order
        for (; r + 3 * (int64_t)rl < rend; r += 4 * (int64_t)rl) {
            float v[4][VEC];
#pragma unroll
            for (int u = 0; u < 4; ++u) Vec<T, VEC>::load(base + (r + u * (int64_t)rl) * ld, v[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int i = 0; i < VEC; ++i) { s[i] += v[u][i]; q[i] = fmaf(v[u][i], v[u][i], q[i]); }
        }
        for (; r < rend; r += rl) {
            float v[VEC];
            Vec<T, VEC>::load(base + r * ld, v);
#pragma unroll
            for (int i = 0; i < VEC; ++i) { s[i] += v[i]; q[i] = fmaf(v[i], v[i], q[i]); }
        }
    }
#pragma unroll
    for (int i = 0; i < VEC; ++i) { red[0][tid * VEC + i] = s[i]; red[1][tid * VEC + i] = q[i]; }
    __syncthreads();
    if (r0 == 0 && cv * VEC < C) {
        for (int i = 0; i < VEC; ++i) {
            float ss = 0.f, qq = 0.f;
            for (int r = 0; r < rl; ++r) {
                ss += red[0][(r * cthreads + cl) * VEC + i];
                qq += red[1][(r * cthreads + cl) * VEC + i];
            }
            size_t o = (((size_t)n * chunks + chunk) * C + (size_t)cv * VEC + i) * 2;
            partial[o] = ss;
            partial[o + 1] = qq;
        }
    }
    if (counts && n == 0 && blockIdx.z == 0 && tid == 0) counts[chunk] = (int32_t)(rend - rbeg);
}

// One 256-thread block per (n,c).  The parts carry (sum, sum of squares, count); they are added in
// fp64 in a fixed order (strided per thread, four parts in flight, then a fixed tree over lanes and
// waves), and mean / variance follow from the totals in fp64: with fp32 part sums as the input this
// loses nothing against merging per-part means and second moments.
// NT threads per (sample, channel): 256, or 1024 where there are thousands of parts (the loop over them is a chain of
// strided loads: its length, not the bytes, is what the kernel takes).
template <int NT>
__global__ __launch_bounds__(NT) void stats_finalize_kernel(const float* __restrict__ partial,
                                                            const int32_t* __restrict__ counts, int parts, int C,
                                                            float eps, float* __restrict__ stats, int counts_per_sample) {
    __shared__ double sh[NT / 64][3];
    const int c = blockIdx.x, n = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int32_t* cnt = counts + (counts_per_sample ? (size_t)n * parts : (size_t)0);
    const float2* pp = reinterpret_cast<const float2*>(partial) + (size_t)n * parts * C + c;
    double k = 0.0, sm = 0.0, sq = 0.0;
    int p = tid;
    for (; p + 3 * NT < parts; p += 4 * NT) {
        float2 v[4];
        int32_t kk[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) { v[u] = pp[(size_t)(p + NT * u) * C]; kk[u] = cnt[p + NT * u]; }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (kk[u] > 0) { k += (double)kk[u]; sm += (double)v[u].x; sq += (double)v[u].y; }
    }
    for (; p < parts; p += NT) {
        const float2 v = pp[(size_t)p * C];
        const int32_t kk = cnt[p];
        if (kk > 0) { k += (double)kk; sm += (double)v.x; sq += (double)v.y; }
    }
    for (int off = 32; off > 0; off >>= 1) {
        k += __shfl_down(k, off);
        sm += __shfl_down(sm, off);
        sq += __shfl_down(sq, off);
    }
    if (lane == 0) { sh[wv][0] = k; sh[wv][1] = sm; sh[wv][2] = sq; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < NT / 64; ++w) { k += sh[w][0]; sm += sh[w][1]; sq += sh[w][2]; }
        double mean = 0.0, var = 0.0;
        if (k > 0.0) {
            mean = sm / k;
            var = sq / k - mean * mean;
            if (var < 0.0) var = 0.0;
        }
        stats[((size_t)n * C + c) * 2 + 0] = (float)mean;
        stats[((size_t)n * C + c) * 2 + 1] = (float)(1.0 / sqrt(var + (double)eps));
    }
}

lamp_status launch_stats_finalize(const float* partials, const int32_t* counts, int parts, int N, int C,
                                  float eps, float* stats, hipStream_t s, bool counts_per_sample) {
    if (parts >= 4096)
        hipLaunchKernelGGL(stats_finalize_kernel<1024>, dim3(C, N), dim3(1024), 0, s, partials, counts, parts, C, eps, stats,
                           counts_per_sample ? 1 : 0);
    else
        hipLaunchKernelGGL(stats_finalize_kernel<256>, dim3(C, N), dim3(256), 0, s, partials, counts, parts, C, eps, stats,
                           counts_per_sample ? 1 : 0);
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}

lamp_status launch_stats(const lamp_tensor_desc* zd, const void* z, float eps, float* stats,
                         void* ws, size_t ws_bytes, hipStream_t s) {
    const int64_t V = (int64_t)zd->d * zd->h * zd->w;
    const int chunks = stats_chunks(V);
    if (!ws || ws_bytes < stats_ws_bytes(zd)) return LAMP_ERR_WORKSPACE;
    float* partial = (float*)ws;
    int32_t* counts = (int32_t*)((char*)ws + align_up((size_t)zd->n * chunks * zd->c * 2 * sizeof(float)));
    const int vec = pick_vec(zd->dtype, zd->c, {zd->ldc}, {z});
    LAMP_DISPATCH_TV(zd->dtype, vec, {
        RowMap m = make_rowmap(zd->c, VEC);
        hipLaunchKernelGGL((stats_partial_kernel<T, VEC>), dim3(chunks, zd->n, m.ctiles), dim3(256), 0, s,
                           (const T*)z, zd->ldc, V, zd->c, m.cthreads, m.rl, rows_per_chunk(V), partial, counts);
    });
    LAMP_CHECK_LAUNCH();
    return launch_stats_finalize(partial, counts, chunks, zd->n, zd->c, eps, stats, s);
}

// ---- sum of split-reduction partials -------------------------------------------------------
// z[v][c] = bf16( sum_s zpart[s][v][c] ), splits added in order; the (sum, sum of squares) of the
// rounded values are accumulated for the statistics like stats_partial_kernel does.  C % 8 == 0.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ zpart, int S, int64_t split_stride,
                                                            bf16_t* __restrict__ z, int ldz, bf16_t* __restrict__ z2, int ldz2,
                                                            int zsplit, int64_t V, int C,
                                                            int cthreads, int rl, int rows_per_chunk,
                                                            float* __restrict__ partial, int32_t* __restrict__ counts) {
    __shared__ float red[2][256 * 8];
    const int tid = threadIdx.x;
    const int cl = tid % cthreads, r0 = tid / cthreads;
    const int cv = blockIdx.z * 256 + cl;
    const int chunk = blockIdx.x, n = blockIdx.y, chunks = gridDim.x;
    const int64_t rbeg = (int64_t)chunk * rows_per_chunk;
    int64_t rend = rbeg + rows_per_chunk;
    if (rend > V) rend = V;
    float s[8], q[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) { s[i] = 0.f; q[i] = 0.f; }
    if (r0 < rl && cv * 8 < C) {
        for (int64_t r = rbeg + r0; r < rend; r += rl) {
            const int64_t row = (int64_t)n * V + r;
            const float* src = zpart + row * C + (int64_t)cv * 8;
            float4 a0 = *reinterpret_cast<const float4*>(src), a1 = *reinterpret_cast<const float4*>(src + 4);
            for (int sp = 1; sp < S; ++sp) {
                const float4 b0 = *reinterpret_cast<const float4*>(src + sp * split_stride);
                const float4 b1 = *reinterpret_cast<const float4*>(src + sp * split_stride + 4);
                a0.x += b0.x; a0.y += b0.y; a0.z += b0.z; a0.w += b0.w;
                a1.x += b1.x; a1.y += b1.y; a1.z += b1.z; a1.w += b1.w;
            }
            const float v[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
            uint32_t pk[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) pk[i] = (uint32_t)f2bf(v[2 * i]) | ((uint32_t)f2bf(v[2 * i + 1]) << 16);
            // channels from zsplit on belong to the second output tensor (two-part output)
            bf16_t* dst = cv * 8 < zsplit ? z + row * ldz + (int64_t)cv * 8 : z2 + row * ldz2 + ((int64_t)cv * 8 - zsplit);
            *reinterpret_cast<uint4*>(dst) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float f0 = __uint_as_float(pk[i] << 16), f1 = __uint_as_float(pk[i] & 0xFFFF0000u);
                s[2 * i] += f0; q[2 * i] = fmaf(f0, f0, q[2 * i]);
                s[2 * i + 1] += f1; q[2 * i + 1] = fmaf(f1, f1, q[2 * i + 1]);
            }
        }
    }
    if (!partial) return;
#pragma unroll
    for (int i = 0; i < 8; ++i) { red[0][tid * 8 + i] = s[i]; red[1][tid * 8 + i] = q[i]; }
    __syncthreads();
    if (r0 == 0 && cv * 8 < C) {
        for (int i = 0; i < 8; ++i) {
            float ss = 0.f, qq = 0.f;
            for (int r = 0; r < rl; ++r) {
                ss += red[0][(r * cthreads + cl) * 8 + i];
                qq += red[1][(r * cthreads + cl) * 8 + i];
            }
            size_t o = (((size_t)n * chunks + chunk) * C + (size_t)cv * 8 + i) * 2;
            partial[o] = ss;
            partial[o + 1] = qq;
        }
    }
    if (n == 0 && blockIdx.z == 0 && tid == 0) counts[chunk] = (int32_t)(rend - rbeg);
}

lamp_status launch_splitk_reduce(const float* zpart, int S, const lamp_tensor_desc* zd, void* z, float eps, float* stats,
                                 void* ws, size_t ws_bytes, hipStream_t s, void* z2, int ldz2, int zsplit) {
    const int64_t V = (int64_t)zd->d * zd->h * zd->w;
    const int chunks = stats_chunks(V);
    float* partial = nullptr;
    int32_t* counts = nullptr;
    if (stats) {
        if (!ws || ws_bytes < stats_ws_bytes(zd)) return LAMP_ERR_WORKSPACE;
        partial = (float*)ws;
        counts = (int32_t*)((char*)ws + align_up((size_t)zd->n * chunks * zd->c * 2 * sizeof(float)));
    }
    const RowMap m = make_rowmap(zd->c, 8);
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3(chunks, zd->n, m.ctiles), dim3(256), 0, s, zpart, S,
                       (int64_t)zd->n * V * zd->c, (bf16_t*)z, zd->ldc, (bf16_t*)z2, ldz2, z2 ? zsplit : 0x7fffffff, V, zd->c,
                       m.cthreads, m.rl, rows_per_chunk(V),
                       partial, counts);
    LAMP_CHECK_LAUNCH();
    if (stats) return launch_stats_finalize(partial, counts, chunks, zd->n, zd->c, eps, stats, s);
    return LAMP_OK;
}

// ---- apply ----------------------------------------------------------------------------------
template <typename T, int VEC>
__global__ __launch_bounds__(256) void inorm_apply_kernel(const T* __restrict__ z, int ldz, T* __restrict__ y, int ldy,
                                                          int64_t V, int C, int cthreads, int rl,
                                                          const float* __restrict__ stats,
                                                          const float* __restrict__ gamma, const float* __restrict__ beta) {
    const int tid = threadIdx.x;
    const int cl = tid % cthreads, r0 = tid / cthreads;
    const int cv = blockIdx.z * 256 + cl;
    const int n = blockIdx.y;
    if (r0 >= rl || cv * VEC >= C) return;
    NormIn nm{stats, gamma, beta, C, 1};
    float a[VEC], b[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) norm_coeffs(nm, n, cv * VEC + i, a[i], b[i]);
    const T* zb = z + ((int64_t)n * V) * ldz + (int64_t)cv * VEC;
    T* yb = y + ((int64_t)n * V) * ldy + (int64_t)cv * VEC;
    for (int64_t r = (int64_t)blockIdx.x * rl + r0; r < V; r += (int64_t)gridDim.x * rl) {
        float v[VEC];
        Vec<T, VEC>::load(zb + r * ldz, v);
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            float u = norm_u(v[i], a[i], b[i]);
            v[i] = u > 0.f ? u : 0.f;
        }
        Vec<T, VEC>::store(yb + r * ldy, v);
    }
}

// ---- backward -------------------------------------------------------------------------------
// partial[((n*chunks+chunk)*C + c)*2] = (sum g, sum g*zh) over the chunk's rows.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void inorm_bwd_partial_kernel(const T* __restrict__ dy, int ldg, const T* __restrict__ z,
                                                                int ldz, int64_t V, int C, int cthreads, int rl,
                                                                int rows_per_chunk, const float* __restrict__ stats,
                                                                const float* __restrict__ gamma,
                                                                const float* __restrict__ beta,
                                                                float* __restrict__ partial) {
    __shared__ float red[2][256 * VEC];
    const int tid = threadIdx.x;
    const int cl = tid % cthreads, r0 = tid / cthreads;
    const int cv = blockIdx.z * 256 + cl;
    const int chunk = blockIdx.x, n = blockIdx.y, chunks = gridDim.x;
    const int64_t rbeg = (int64_t)chunk * rows_per_chunk;
    int64_t rend = rbeg + rows_per_chunk;
    if (rend > V) rend = V;
    float s[VEC], q[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) { s[i] = 0.f; q[i] = 0.f; }
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
        const T* gb = dy + ((int64_t)n * V) * ldg + (int64_t)cv * VEC;
        auto add_row = [&](const float (&v)[VEC], const float (&g)[VEC]) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                float u = norm_u(v[i], a[i], b[i]);
                float gg = u > 0.f ? g[i] : 0.f;
                float zh = (v[i] - mean[i]) * rstd[i];
                s[i] += gg;
                q[i] = fmaf(gg, zh, q[i]);
            }
        };
        int64_t r = rbeg + r0;
        // four rows in flight; the additions keep the row order
        for (; r + 3 * (int64_t)rl < rend; r += 4 * (int64_t)rl) {
            float v[4][VEC], g[4][VEC];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                Vec<T, VEC>::load(zb + (r + u * (int64_t)rl) * ldz, v[u]);
                Vec<T, VEC>::load(gb + (r + u * (int64_t)rl) * ldg, g[u]);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) add_row(v[u], g[u]);
        }
        for (; r < rend; r += rl) {
            float v[VEC], g[VEC];
            Vec<T, VEC>::load(zb + r * ldz, v);
            Vec<T, VEC>::load(gb + r * ldg, g);
            add_row(v, g);
        }
    }
#pragma unroll
    for (int i = 0; i < VEC; ++i) { red[0][tid * VEC + i] = s[i]; red[1][tid * VEC + i] = q[i]; }
    __syncthreads();
    if (r0 == 0 && cv * VEC < C) {
        for (int i = 0; i < VEC; ++i) {
            float ss = 0.f, qq = 0.f;
            for (int r = 0; r < rl; ++r) {
                ss += red[0][(r * cthreads + cl) * VEC + i];
                qq += red[1][(r * cthreads + cl) * VEC + i];
            }
            size_t o = (((size_t)n * chunks + chunk) * C + (size_t)cv * VEC + i) * 2;
            partial[o] = ss;
            partial[o + 1] = qq;
        }
    }
}

// sums[n][c][2] = (sum g, sum g*zh) over all parts, fp64, fixed order (strided per thread with four
// parts in flight, then a fixed tree over lanes and waves).
// zstats != nullptr: the second partial sum is over g*z (raw z, from the data-gradient epilogue) and is turned into
// the sum over g*zhat here, in fp64: rstd * (sum g*z - mean * sum g).
__global__ __launch_bounds__(256) void inorm_bwd_finalize_kernel(const float* __restrict__ partial, int parts, int C,
                                                                 float* __restrict__ sums, const float* __restrict__ zstats) {
    __shared__ double sh[4][2];
    const int c = blockIdx.x, n = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const float2* pp = reinterpret_cast<const float2*>(partial) + (size_t)n * parts * C + c;
    double s = 0.0, q = 0.0;
    int p = tid;
    for (; p + 768 < parts; p += 1024) {
        float2 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = pp[(size_t)(p + 256 * u) * C];
#pragma unroll
        for (int u = 0; u < 4; ++u) { s += (double)v[u].x; q += (double)v[u].y; }
    }
    for (; p < parts; p += 256) {
        const float2 v = pp[(size_t)p * C];
        s += (double)v.x;
        q += (double)v.y;
    }
    for (int off = 32; off > 0; off >>= 1) {
        s += __shfl_down(s, off);
        q += __shfl_down(q, off);
    }
    if (lane == 0) { sh[wv][0] = s; sh[wv][1] = q; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w) { s += sh[w][0]; q += sh[w][1]; }
        if (zstats) q = (double)zstats[((size_t)n * C + c) * 2 + 1] * (q - (double)zstats[((size_t)n * C + c) * 2 + 0] * s);
        sums[((size_t)n * C + c) * 2 + 0] = (float)s;
        sums[((size_t)n * C + c) * 2 + 1] = (float)q;
    }
}

__global__ void inorm_dgb_kernel(const float* __restrict__ sums, int N, int C, float* dgamma, float* dbeta,
                                 float beta_acc) {
    int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    double s = 0.0, q = 0.0;
    for (int n = 0; n < N; ++n) {
        s += (double)sums[((size_t)n * C + c) * 2 + 0];
        q += (double)sums[((size_t)n * C + c) * 2 + 1];
    }
    if (dbeta) dbeta[c] = (beta_acc != 0.f ? beta_acc * dbeta[c] : 0.f) + (float)s;
    if (dgamma) dgamma[c] = (beta_acc != 0.f ? beta_acc * dgamma[c] : 0.f) + (float)q;
}

template <typename T, int VEC>
__global__ __launch_bounds__(256) void inorm_bwd_apply_kernel(const T* __restrict__ dy, int ldg, const T* __restrict__ z,
                                                              int ldz, T* __restrict__ dz, int ldo, int64_t V, int C,
                                                              int cthreads, int rl, const float* __restrict__ stats,
                                                              const float* __restrict__ gamma,
                                                              const float* __restrict__ beta,
                                                              const float* __restrict__ sums) {
    const int tid = threadIdx.x;
    const int cl = tid % cthreads, r0 = tid / cthreads;
    const int cv = blockIdx.z * 256 + cl;
    const int n = blockIdx.y;
    if (r0 >= rl || cv * VEC >= C) return;
    NormIn nm{stats, gamma, beta, C, 1};
    float a[VEC], b[VEC], mean[VEC], rstd[VEC], c1[VEC], c2[VEC];
    const float invV = 1.0f / (float)V;
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        norm_coeffs(nm, n, cv * VEC + i, a[i], b[i]);
        mean[i] = stats[((size_t)n * C + cv * VEC + i) * 2];
        rstd[i] = stats[((size_t)n * C + cv * VEC + i) * 2 + 1];
        c1[i] = sums[((size_t)n * C + cv * VEC + i) * 2] * invV;
        c2[i] = sums[((size_t)n * C + cv * VEC + i) * 2 + 1] * invV;
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
            float u = norm_u(v[i], a[i], b[i]);
            float gg = u > 0.f ? g[i] : 0.f;
            float zh = (v[i] - mean[i]) * rstd[i];
            v[i] = a[i] * (gg - c1[i] - zh * c2[i]);
        }
        Vec<T, VEC>::store(ob + r * ldo, v);
    }
}

static int apply_blocks(int64_t V, int rl) {
    int64_t b = (V + rl - 1) / rl;
    int64_t cap = 256 * 16;
    b = (b + 3) / 4;  // a few rows per thread
    if (b < 1) b = 1;
    return (int)(b > cap ? cap : b);
}

}  // namespace lamp

using namespace lamp;

extern "C" size_t lamp_inorm_relu_workspace_bytes(const lamp_tensor_desc* zd) {
    if (!desc_ok(zd)) return 0;
    return stats_ws_bytes(zd);
}

extern "C" lamp_status lamp_inorm_relu(const lamp_tensor_desc* zd, const void* z, const float* gamma,
                                       const float* beta, float eps, const lamp_tensor_desc* yd, void* y,
                                       float* stats, int stats_given, void* ws, size_t ws_bytes, void* stream) {
    if (!zd || !yd || !z || !y || !stats) return LAMP_ERR_NULL;
    if (!desc_ok(zd) || !desc_ok(yd) || !same_space(zd, yd) || zd->c != yd->c) return LAMP_ERR_SHAPE;
    if (zd->dtype != yd->dtype) return LAMP_ERR_DTYPE;
    if (!(eps >= 0.f)) return LAMP_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    if (!stats_given) {
        if (!ws || ws_bytes < stats_ws_bytes(zd)) return LAMP_ERR_WORKSPACE;
        lamp_status st = launch_stats(zd, z, eps, stats, ws, ws_bytes, s);
        if (st != LAMP_OK) return st;
    }
    const int64_t V = (int64_t)zd->d * zd->h * zd->w;
    const int vec = pick_vec(zd->dtype, zd->c, {zd->ldc, yd->ldc}, {z, y});
    LAMP_DISPATCH_TV(zd->dtype, vec, {
        RowMap m = make_rowmap(zd->c, VEC);
        hipLaunchKernelGGL((inorm_apply_kernel<T, VEC>), dim3(apply_blocks(V, m.rl), zd->n, m.ctiles), dim3(256), 0, s,
                           (const T*)z, zd->ldc, (T*)y, yd->ldc, V, zd->c, m.cthreads, m.rl, stats, gamma, beta);
    });
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}

extern "C" lamp_status lamp_inorm_relu_noalloc(const lamp_tensor_desc* zd, const void* z, const float* gamma,
                                               const float* beta, float eps, const lamp_tensor_desc* yd, void* y,
                                               float* stats, void* stream) {
    if (!zd || !yd || !z || !y || !stats) return LAMP_ERR_NULL;
    if (!desc_ok(zd) || !desc_ok(yd)) return LAMP_ERR_SHAPE;
    if (stats_ws_bytes(zd) > (size_t)LAMP_NOALLOC_SCRATCH_BYTES) return LAMP_ERR_WORKSPACE;   // beyond the fixed scratch
    void* ptr = nullptr;
    lamp_status st = noalloc_scratch(&ptr);
    if (st != LAMP_OK) return st;
    // Nothing in the scratch has to start at zero: the statistics pass writes every partial and every count
    // that its second stage reads, so what the previous call left there is never seen.
    return lamp_inorm_relu(zd, z, gamma, beta, eps, yd, y, stats, 0, ptr, (size_t)LAMP_NOALLOC_SCRATCH_BYTES, stream);
}

extern "C" size_t lamp_inorm_relu_bwd_workspace_bytes(const lamp_tensor_desc* zd) {
    if (!desc_ok(zd)) return 0;
    int64_t V = (int64_t)zd->d * zd->h * zd->w;
    int ch = stats_chunks(V);
    return align_up((size_t)zd->n * ch * zd->c * 2 * sizeof(float)) + align_up((size_t)zd->n * zd->c * 2 * sizeof(float));
}

extern "C" lamp_status lamp_inorm_relu_bwd(const lamp_tensor_desc* dyd, const void* dy, const lamp_tensor_desc* zd,
                                           const void* z, const float* stats, const float* gamma, const float* beta,
                                           const lamp_tensor_desc* dzd, void* dz, float* dgamma, float* dbeta,
                                           float beta_acc, void* ws, size_t ws_bytes, void* stream) {
    if (!dyd || !zd || !dzd || !dy || !z || !stats || !dz) return LAMP_ERR_NULL;
    if (!desc_ok(dyd) || !desc_ok(zd) || !desc_ok(dzd) || !same_space(zd, dyd) || !same_space(zd, dzd) ||
        zd->c != dyd->c || zd->c != dzd->c)
        return LAMP_ERR_SHAPE;
    if (zd->dtype != dyd->dtype || zd->dtype != dzd->dtype) return LAMP_ERR_DTYPE;
    if (beta_acc != 0.f && beta_acc != 1.f) return LAMP_ERR_SHAPE;
    if (!ws || ws_bytes < lamp_inorm_relu_bwd_workspace_bytes(zd)) return LAMP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int64_t V = (int64_t)zd->d * zd->h * zd->w;
    const int chunks = stats_chunks(V);
    float* partial = (float*)ws;
    float* sums = (float*)((char*)ws + align_up((size_t)zd->n * chunks * zd->c * 2 * sizeof(float)));
    const int vec = pick_vec(zd->dtype, zd->c, {zd->ldc, dyd->ldc, dzd->ldc}, {z, dy, dz});
    LAMP_DISPATCH_TV(zd->dtype, vec, {
        RowMap m = make_rowmap(zd->c, VEC);
        hipLaunchKernelGGL((inorm_bwd_partial_kernel<T, VEC>), dim3(chunks, zd->n, m.ctiles), dim3(256), 0, s,
                           (const T*)dy, dyd->ldc, (const T*)z, zd->ldc, V, zd->c, m.cthreads, m.rl, rows_per_chunk(V),
                           stats, gamma, beta, partial);
    });
    LAMP_CHECK_LAUNCH();
    hipLaunchKernelGGL(inorm_bwd_finalize_kernel, dim3(zd->c, zd->n), dim3(256), 0, s, partial, chunks, zd->c, sums,
                       (const float*)nullptr);
    LAMP_CHECK_LAUNCH();
    return launch_inorm_bwd_apply(dyd, dy, zd, z, stats, gamma, beta, sums, dzd, dz, dgamma, dbeta, beta_acc, s);
}

lamp_status lamp::launch_bsum_finalize(const float* partial, int parts, int N, int C, const float* zstats, float* sums, hipStream_t s) {
    hipLaunchKernelGGL(inorm_bwd_finalize_kernel, dim3(C, N), dim3(256), 0, s, partial, parts, C, sums, zstats);
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}

lamp_status lamp::launch_inorm_bwd_apply(const lamp_tensor_desc* dyd, const void* dy, const lamp_tensor_desc* zd, const void* z,
                                   const float* stats, const float* gamma, const float* beta, const float* sums,
                                   const lamp_tensor_desc* dzd, void* dz, float* dgamma, float* dbeta, float beta_acc,
                                   hipStream_t s) {
    const int64_t V = (int64_t)zd->d * zd->h * zd->w;
    const int vec = pick_vec(zd->dtype, zd->c, {zd->ldc, dyd->ldc, dzd->ldc}, {z, dy, dz});
    if (dgamma || dbeta) {
        hipLaunchKernelGGL(inorm_dgb_kernel, dim3(cdiv(zd->c, 64)), dim3(64), 0, s, sums, zd->n, zd->c, dgamma, dbeta,
                           beta_acc);
        LAMP_CHECK_LAUNCH();
    }
    LAMP_DISPATCH_TV(zd->dtype, vec, {
        RowMap m = make_rowmap(zd->c, VEC);
        hipLaunchKernelGGL((inorm_bwd_apply_kernel<T, VEC>), dim3(apply_blocks(V, m.rl), zd->n, m.ctiles), dim3(256), 0,
                           s, (const T*)dy, dyd->ldc, (const T*)z, zd->ldc, (T*)dz, dzd->ldc, V, zd->c, m.cthreads,
                           m.rl, stats, gamma, beta, sums);
    });
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}
