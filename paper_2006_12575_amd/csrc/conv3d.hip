// 3x3x3 convolution: public entry points, argument checking, kernel selection, and the generic
// direct kernels (any dtype / channel count) that serve the fp32 path and odd channel counts.
// Shapes with channel counts in multiples of 32 in bf16 go to the matrix-core kernels.
#include "internal.h"

namespace lamp {

// out[v][oc] = bias[oc] + sum_t sum_ic in[v + t - 1][ic] * Wv(oc,t,ic)
//   forward : Wv(oc,t,ic) = W[oc][t][ic]          (W is [Cout][27][Cin])
//   dgrad   : Wv(oc,t,ic) = W[ic][26-t][oc]       (W is [Cin][27][Cout]: flipped taps, swapped roles)
template <typename T, bool DGRAD>
__global__ __launch_bounds__(256) void conv3d_direct_kernel(const T* __restrict__ x, int ldx, NormIn nm,
                                                            const T* __restrict__ w, const float* __restrict__ bias,
                                                            T* __restrict__ z, int ldz, int N, int D, int H, int W,
                                                            int Cin, int Cout, int ocT, int vpb) {
    const int oc = blockIdx.y * ocT + threadIdx.x % ocT;
    const int vl = threadIdx.x / ocT;
    if (vl >= vpb || oc >= Cout) return;
    const int64_t total = (int64_t)N * D * H * W;
    const int64_t v = (int64_t)blockIdx.x * vpb + vl;
    if (v >= total) return;
    int wv = (int)(v % W);
    int64_t r = v / W;
    int h = (int)(r % H);
    r /= H;
    int d = (int)(r % D);
    int n = (int)(r / D);
    float acc = bias ? bias[oc] : 0.f;
    for (int t = 0; t < 27; ++t) {
        int kd = t / 9, kh = (t / 3) % 3, kw = t % 3;
        int id = d + kd - 1, ih = h + kh - 1, iw = wv + kw - 1;
        if (id < 0 || id >= D || ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
        const T* xp = x + ((((int64_t)n * D + id) * H + ih) * W + iw) * ldx;
        if (DGRAD) {
            const T* wp = w + (int64_t)(26 - t) * Cout + oc;
            for (int ic = 0; ic < Cin; ++ic)
                acc = fmaf(load_norm(xp + ic, nm, n, ic), io<T>::ld(wp + (int64_t)ic * 27 * Cout), acc);
        } else {
            const T* wp = w + ((int64_t)oc * 27 + t) * Cin;
            for (int ic = 0; ic < Cin; ++ic)
                acc = fmaf(load_norm(xp + ic, nm, n, ic), io<T>::ld(wp + ic), acc);
        }
    }
    io<T>::st(z + v * ldz + oc, acc);
}

// part[s][o] for o = (co*27 + t)*Ci + ci : sum over the voxels of split s.
template <typename T>
__global__ __launch_bounds__(256) void conv3d_wgrad_direct_kernel(const T* __restrict__ x, int ldx, NormIn nm,
                                                                  const T* __restrict__ dz, int ldz,
                                                                  float* __restrict__ part, int N, int D, int H, int W,
                                                                  int Ci, int Co, int64_t vps) {
    const int64_t O = (int64_t)Co * 27 * Ci;
    const int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (o >= O) return;
    const int ci = (int)(o % Ci);
    const int t = (int)((o / Ci) % 27);
    const int co = (int)(o / ((int64_t)27 * Ci));
    const int kd = t / 9 - 1, kh = (t / 3) % 3 - 1, kw = t % 3 - 1;
    const int64_t total = (int64_t)N * D * H * W;
    int64_t v0 = (int64_t)blockIdx.y * vps, v1 = v0 + vps;
    if (v1 > total) v1 = total;
    int wv = (int)(v0 % W);
    int64_t r = v0 / W;
    int h = (int)(r % H);
    r /= H;
    int d = (int)(r % D);
    int n = (int)(r / D);
    float acc = 0.f;
    for (int64_t v = v0; v < v1; ++v) {
        int id = d + kd, ih = h + kh, iw = wv + kw;
        if (id >= 0 && id < D && ih >= 0 && ih < H && iw >= 0 && iw < W) {
            const T* xp = x + ((((int64_t)n * D + id) * H + ih) * W + iw) * ldx + ci;
            acc = fmaf(io<T>::ld(dz + v * ldz + co), load_norm(xp, nm, n, ci), acc);
        }
        if (++wv == W) { wv = 0; if (++h == H) { h = 0; if (++d == D) { d = 0; ++n; } } }
    }
    part[(int64_t)blockIdx.y * O + o] = acc;
}

// ---- single-input-channel first layer (the network input is one CT channel), bf16 ----------------
// Forward: one thread per output voxel computes all Cout channels from its 27 neighbours; the op
// is bound by writing the output (2*Cout bytes per voxel against 2 bytes read).
__global__ __launch_bounds__(256) void conv3d_cin1_fwd_kernel(const bf16_t* __restrict__ x, int ldx,
                                                              const bf16_t* __restrict__ w, bf16_t* __restrict__ z, int ldz,
                                                              int N, int D, int H, int W, int Cout) {
    __shared__ float wsh[27 * 128];  // [tap][co]
    for (int i = threadIdx.x; i < 27 * Cout; i += 256) {
        const int co = i / 27, t = i - co * 27;
        wsh[t * Cout + co] = bf2f(w[i]);
    }
    __syncthreads();
    const int64_t total = (int64_t)N * D * H * W;
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v >= total) return;
    const int wv = (int)(v % W);
    int64_t r = v / W;
    const int h = (int)(r % H);
    r /= H;
    const int d = (int)(r % D);
    const int n = (int)(r / D);
    float xv[27];
#pragma unroll
    for (int t = 0; t < 27; ++t) {
        const int id = d + t / 9 - 1, ih = h + (t / 3) % 3 - 1, iw = wv + t % 3 - 1;
        const bool in = id >= 0 && id < D && ih >= 0 && ih < H && iw >= 0 && iw < W;
        xv[t] = in ? bf2f(x[((((int64_t)n * D + id) * H + ih) * W + iw) * ldx]) : 0.f;
    }
    bf16_t* zp = z + v * ldz;
    for (int c8 = 0; c8 < Cout; c8 += 8) {
        float acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
        for (int t = 0; t < 27; ++t)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = fmaf(xv[t], wsh[t * Cout + c8 + e], acc[e]);
        uint32_t pk[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) pk[e] = (uint32_t)f2bf(acc[2 * e]) | ((uint32_t)f2bf(acc[2 * e + 1]) << 16);
        *reinterpret_cast<uint4*>(zp + c8) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
    }
}

// Forward for Cin == 1 with C_out % 32 == 0 on the matrix cores: z^T[co][voxel] = W[co][tap] * X27^T[tap][voxel],
// taps (27, padded to 32) as the reduction dimension.  A = weights (kept in registers), B = the gathered
// neighbours of 32 consecutive voxels (8 two-byte loads per lane and k-block, served by the caches); every
// lane ends with 4 consecutive channels per register group of its voxel and stores them as 8 bytes.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 c1_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float c1_f32x16;
__global__ __launch_bounds__(256, 4) void conv3d_cin1_fwd_mfma_kernel(const bf16_t* __restrict__ x, int ldx,
                                                                      const bf16_t* __restrict__ w, bf16_t* __restrict__ z,
                                                                      int ldz, int N, int D, int H, int W, int Cout) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, l32 = lane & 31, half = lane >> 5;
    const int CB = Cout >> 5;
    c1_bf16x8 a[4][2];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            uint32_t r[4] = {0, 0, 0, 0};
            if (cb < CB) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int t = 16 * kb + 8 * half + e;
                    const uint32_t b = t < 27 ? (uint32_t)w[(size_t)(32 * cb + l32) * 27 + t] : 0u;
                    r[e >> 1] |= b << (16 * (e & 1));
                }
            }
            a[cb][kb] = __builtin_bit_cast(c1_bf16x8, make_uint4(r[0], r[1], r[2], r[3]));
        }
    const int64_t total = (int64_t)N * D * H * W;
    const int64_t groups = (total + 31) / 32;
    for (int64_t g = (int64_t)blockIdx.x * 4 + wv; g < groups; g += (int64_t)gridDim.x * 4) {
        const int64_t v = g * 32 + l32;
        const bool valid = v < total;
        const int64_t vc = valid ? v : 0;
        const int wq = (int)(vc % W);
        int64_t rr = vc / W;
        const int h = (int)(rr % H);
        rr /= H;
        const int d = (int)(rr % D);
        const int n = (int)(rr / D);
        c1_bf16x8 b[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            uint32_t r[4] = {0, 0, 0, 0};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int t = 16 * kb + 8 * half + e;
                const int id = d + t / 9 - 1, ih = h + (t / 3) % 3 - 1, iw = wq + t % 3 - 1;
                const bool in = valid && t < 27 && id >= 0 && id < D && ih >= 0 && ih < H && iw >= 0 && iw < W;
                const uint32_t xv = in ? (uint32_t)x[((((int64_t)n * D + id) * H + ih) * W + iw) * ldx] : 0u;
                r[e >> 1] |= xv << (16 * (e & 1));
            }
            b[kb] = __builtin_bit_cast(c1_bf16x8, make_uint4(r[0], r[1], r[2], r[3]));
        }
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) {
            if (cb < CB) {
                c1_f32x16 acc;
#pragma unroll
                for (int q = 0; q < 16; ++q) acc[q] = 0.f;
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cb][0], b[0], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cb][1], b[1], acc, 0, 0, 0);
                if (valid) {
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        const uint32_t p0 = (uint32_t)f2bf(acc[rg * 4 + 0]) | ((uint32_t)f2bf(acc[rg * 4 + 1]) << 16);
                        const uint32_t p1 = (uint32_t)f2bf(acc[rg * 4 + 2]) | ((uint32_t)f2bf(acc[rg * 4 + 3]) << 16);
                        *reinterpret_cast<uint2*>(z + v * ldz + 32 * cb + 8 * rg + 4 * half) = make_uint2(p0, p1);
                    }
                }
            }
        }
    }
}

// Weight gradient for Cin == 1: dW[co][tap] = sum_v dz[v][co] * x[v + tap], as a matrix-core product
// with the voxels as the reduction dimension.  Per step a wave multiplies A = dz^T (32 channels x 16
// voxels of one W-row) by B = the gathered neighbours (16 voxels x 32 taps, taps 27..31 zero); both
// fragments come straight from global memory (dz is read once, x is cache-resident).  Every wave
// owns a run of 16-voxel groups and writes its own partial [Co][27] slab.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
struct U16x8 { unsigned short e[8]; };

__global__ __launch_bounds__(256) void conv3d_cin1_wgrad_kernel(const bf16_t* __restrict__ x, int ldx,
                                                                const bf16_t* __restrict__ dz, int lddz,
                                                                float* __restrict__ part, int N, int D, int H, int W, int Co,
                                                                int64_t groups, int gpw) {
    const int lane = threadIdx.x & 63, l32 = lane & 31, kg = lane >> 5;
    const int64_t wid = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int cob = blockIdx.y * 32;
    const int tap = l32;
    const int kd = tap / 9 - 1, kh = (tap / 3) % 3 - 1, kw = tap % 3 - 1;
    int64_t g0 = wid * gpw, g1 = g0 + gpw;
    if (g1 > groups) g1 = groups;
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    for (int64_t g = g0; g < g1; ++g) {
        const int64_t v = g * 16 + 8 * kg;  // the lane's 8 voxels v..v+7 lie in one W-row
        const int w0 = (int)(v % W);
        int64_t r = v / W;
        const int h = (int)(r % H);
        r /= H;
        const int d = (int)(r % D);
        const int n = (int)(r / D);
        U16x8 a, b;
        const bf16_t* dp = dz + v * lddz + cob + l32;
#pragma unroll
        for (int e = 0; e < 8; ++e) a.e[e] = dp[(int64_t)e * lddz];
        const int id = d + kd, ih = h + kh;
        const bool rowok = tap < 27 && id >= 0 && id < D && ih >= 0 && ih < H;
        const int64_t base = rowok ? (((int64_t)n * D + id) * H + ih) * W : 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int iw = w0 + e + kw;
            const bool ok = rowok && iw >= 0 && iw < W;
            b.e[e] = ok ? x[(base + iw) * ldx] : (bf16_t)0;
        }
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0,
                                                      0);
    }
    if (tap < 27) {
        float* pb = part + wid * Co * 27;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int co = cob + 8 * (r / 4) + 4 * kg + (r % 4);
            pb[(int64_t)co * 27 + tap] = acc[r];
        }
    }
}

static bool cin1_fwd_ok(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd, const lamp_norm_in* xnorm, const float* bias,
                        const void* z) {
    const bool nm = xnorm && xnorm->mean_rstd && xnorm->c_norm > 0;
    return xd->dtype == LAMP_BF16 && xd->c == 1 && !nm && !bias && zd->c % 8 == 0 && zd->c <= 128 && zd->ldc % 8 == 0 &&
           aligned16(z);
}
static bool cin1_wgrad_ok(const lamp_tensor_desc* xd, const lamp_tensor_desc* dzd, const lamp_norm_in* xnorm) {
    const bool nm = xnorm && xnorm->mean_rstd && xnorm->c_norm > 0;
    return xd->dtype == LAMP_BF16 && xd->c == 1 && !nm && dzd->c % 32 == 0 && xd->w % 16 == 0;
}
// thread blocks (4 waves, one partial slab per wave) of the Cin == 1 weight gradient
static int cin1_wgrad_blocks(int64_t V) {
    int64_t b = (V / 16 + 3) / 4;
    return (int)(b > 512 ? 512 : (b < 1 ? 1 : b));
}

static int wgrad_splits(int64_t V, int64_t O) {
    int64_t s = (V + 255) / 256;
    int64_t cap = (int64_t)(32u << 20) / (O * 4);
    if (cap < 1) cap = 1;
    if (s > cap) s = cap;
    if (s > 8192) s = 8192;
    if (s < 1) s = 1;
    return (int)s;
}

static lamp_status check_conv_pair(const lamp_tensor_desc* a, const void* pa, const lamp_tensor_desc* b, const void* pb) {
    if (!a || !b || !pa || !pb) return LAMP_ERR_NULL;
    if (!desc_ok(a) || !desc_ok(b) || !same_space(a, b)) return LAMP_ERR_SHAPE;
    if (a->dtype != b->dtype) return LAMP_ERR_DTYPE;
    if (a->dtype == LAMP_BF16 && (!aligned16(pa) || !aligned16(pb))) return LAMP_ERR_ALIGN;
    return LAMP_OK;
}

template <bool DGRAD>
static lamp_status launch_direct(const lamp_tensor_desc* xd, const void* x, NormIn nm, const void* w, const float* bias,
                                 const lamp_tensor_desc* zd, void* z, hipStream_t s) {
    const int Cout = zd->c, Cin = xd->c;
    const int ocT = Cout < 256 ? Cout : 256;
    const int vpb = 256 / ocT;
    const int64_t total = nvox(zd);
    dim3 grid(cdiv(total, vpb), cdiv(Cout, ocT));
    if (xd->dtype == LAMP_BF16)
        hipLaunchKernelGGL((conv3d_direct_kernel<bf16_t, DGRAD>), grid, dim3(256), 0, s, (const bf16_t*)x, xd->ldc, nm,
                           (const bf16_t*)w, bias, (bf16_t*)z, zd->ldc, zd->n, zd->d, zd->h, zd->w, Cin, Cout, ocT, vpb);
    else
        hipLaunchKernelGGL((conv3d_direct_kernel<float, DGRAD>), grid, dim3(256), 0, s, (const float*)x, xd->ldc, nm,
                           (const float*)w, bias, (float*)z, zd->ldc, zd->n, zd->d, zd->h, zd->w, Cin, Cout, ocT, vpb);
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}

}  // namespace lamp

using namespace lamp;

extern "C" size_t lamp_conv3d_fwd_workspace_bytes(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd, int want_stats) {
    if (!desc_ok(xd) || !desc_ok(zd)) return 0;
    size_t a = want_stats ? stats_ws_bytes(zd) : 0;
    size_t b = mfma_conv_ws_bytes(xd, zd, want_stats);
    return a > b ? a : b;
}

extern "C" lamp_status lamp_conv3d_fwd(const lamp_tensor_desc* xd, const void* x, const lamp_norm_in* xnorm, const void* w,
                                       const float* bias, const lamp_tensor_desc* zd, void* z, float* stats_out, float eps,
                                       void* ws, size_t ws_bytes, void* stream) {
    lamp_status st = check_conv_pair(xd, x, zd, z);
    if (st != LAMP_OK) return st;
    if (!w) return LAMP_ERR_NULL;
    if ((st = norm_ok(xnorm, xd)) != LAMP_OK) return st;
    if (stats_out && !(eps >= 0.f)) return LAMP_ERR_SHAPE;
    if (ws_bytes < lamp_conv3d_fwd_workspace_bytes(xd, zd, stats_out != nullptr) || (ws_bytes && !ws))
        return LAMP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    if (mfma_conv_supported(xd, zd, xnorm, bias))
        return mfma_conv_fwd(xd, x, w, false, zd, z, stats_out, eps, ws, ws_bytes, s);
    if (cin1_fwd_ok(xd, zd, xnorm, bias, z)) {
        if (zd->c % 32 == 0) {
            const int64_t wg = (nvox(zd) + 127) / 128;
            const dim3 grid((unsigned)(wg > 8192 ? 8192 : wg));
            hipLaunchKernelGGL(conv3d_cin1_fwd_mfma_kernel, grid, dim3(256), 0, s, (const bf16_t*)x, xd->ldc, (const bf16_t*)w,
                               (bf16_t*)z, zd->ldc, zd->n, zd->d, zd->h, zd->w, zd->c);
        } else {
            hipLaunchKernelGGL(conv3d_cin1_fwd_kernel, dim3(cdiv(nvox(zd), 256)), dim3(256), 0, s, (const bf16_t*)x, xd->ldc,
                               (const bf16_t*)w, (bf16_t*)z, zd->ldc, zd->n, zd->d, zd->h, zd->w, zd->c);
        }
        LAMP_CHECK_LAUNCH();
    } else {
        st = launch_direct<false>(xd, x, make_norm(xnorm), w, bias, zd, z, s);
        if (st != LAMP_OK) return st;
    }
    if (stats_out) return launch_stats(zd, z, eps, stats_out, ws, ws_bytes, s);
    return LAMP_OK;
}

extern "C" size_t lamp_conv3d_dgrad_workspace_bytes(const lamp_tensor_desc* dzd, const lamp_tensor_desc* dxd) {
    if (!desc_ok(dzd) || !desc_ok(dxd)) return 0;
    return mfma_conv_ws_bytes(dzd, dxd, 0);
}

extern "C" lamp_status lamp_conv3d_dgrad(const lamp_tensor_desc* dzd, const void* dz, const void* w,
                                         const lamp_tensor_desc* dxd, void* dx, void* ws, size_t ws_bytes, void* stream) {
    lamp_status st = check_conv_pair(dzd, dz, dxd, dx);
    if (st != LAMP_OK) return st;
    if (!w) return LAMP_ERR_NULL;
    if (ws_bytes < lamp_conv3d_dgrad_workspace_bytes(dzd, dxd) || (ws_bytes && !ws)) return LAMP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    if (mfma_conv_supported(dzd, dxd, nullptr, nullptr))
        return mfma_conv_fwd(dzd, dz, w, true, dxd, dx, nullptr, 0.f, ws, ws_bytes, s);
    return launch_direct<true>(dzd, dz, make_norm(nullptr), w, nullptr, dxd, dx, s);
}

extern "C" size_t lamp_conv3d_wgrad_workspace_bytes(const lamp_tensor_desc* xd, const lamp_tensor_desc* dzd) {
    if (!desc_ok(xd) || !desc_ok(dzd)) return 0;
    const int64_t O = (int64_t)dzd->c * 27 * xd->c;
    size_t a = align_up((size_t)wgrad_splits(nvox(xd), O) * O * sizeof(float));
    size_t b = mfma_wgrad_ws_bytes(xd, dzd);
    size_t c = colsum_ws_bytes(nvox(dzd), dzd->c);
    if (cin1_wgrad_ok(xd, dzd, nullptr)) {
        const size_t e = align_up((size_t)cin1_wgrad_blocks(nvox(xd)) * 4 * dzd->c * 27 * sizeof(float));
        if (e > a) a = e;
    }
    return (a > b ? a : b) + c;
}

extern "C" lamp_status lamp_conv3d_wgrad(const lamp_tensor_desc* xd, const void* x, const lamp_norm_in* xnorm,
                                         const lamp_tensor_desc* dzd, const void* dz, float* dw, float* dbias, float beta,
                                         void* ws, size_t ws_bytes, void* stream) {
    lamp_status st = check_conv_pair(xd, x, dzd, dz);
    if (st != LAMP_OK) return st;
    if (!dw) return LAMP_ERR_NULL;
    if ((st = norm_ok(xnorm, xd)) != LAMP_OK) return st;
    if (beta != 0.f && beta != 1.f) return LAMP_ERR_SHAPE;
    if (!ws || ws_bytes < lamp_conv3d_wgrad_workspace_bytes(xd, dzd)) return LAMP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int64_t O = (int64_t)dzd->c * 27 * xd->c;
    const size_t cs = colsum_ws_bytes(nvox(dzd), dzd->c);
    char* wsb = (char*)ws;
    if (dbias) {
        st = launch_colsum(dz, dzd->dtype, nvox(dzd), dzd->c, dzd->ldc, dbias, beta, wsb + (ws_bytes - cs), cs, s);
        if (st != LAMP_OK) return st;
    }
    if (mfma_wgrad_supported(xd, dzd, xnorm)) return mfma_wgrad(xd, x, dzd, dz, dw, beta, ws, ws_bytes - cs, s);
    if (cin1_wgrad_ok(xd, dzd, xnorm)) {
        const int64_t groups = nvox(xd) / 16;
        const int blocks = cin1_wgrad_blocks(nvox(xd));
        const int gpw = (int)((groups + blocks * 4 - 1) / (blocks * 4));
        hipLaunchKernelGGL(conv3d_cin1_wgrad_kernel, dim3(blocks, dzd->c / 32), dim3(256), 0, s, (const bf16_t*)x, xd->ldc,
                           (const bf16_t*)dz, dzd->ldc, (float*)ws, xd->n, xd->d, xd->h, xd->w, dzd->c, groups, gpw);
        LAMP_CHECK_LAUNCH();
        return launch_reduce_partials((const float*)ws, blocks * 4, (int64_t)dzd->c * 27, dw, beta, s);
    }
    const int64_t V = nvox(xd);
    const int S = wgrad_splits(V, O);
    const int64_t vps = (V + S - 1) / S;
    float* part = (float*)ws;
    dim3 grid(cdiv(O, 256), S);
    NormIn nm = make_norm(xnorm);
    if (xd->dtype == LAMP_BF16)
        hipLaunchKernelGGL((conv3d_wgrad_direct_kernel<bf16_t>), grid, dim3(256), 0, s, (const bf16_t*)x, xd->ldc, nm,
                           (const bf16_t*)dz, dzd->ldc, part, xd->n, xd->d, xd->h, xd->w, xd->c, dzd->c, vps);
    else
        hipLaunchKernelGGL((conv3d_wgrad_direct_kernel<float>), grid, dim3(256), 0, s, (const float*)x, xd->ldc, nm,
                           (const float*)dz, dzd->ldc, part, xd->n, xd->d, xd->h, xd->w, xd->c, dzd->c, vps);
    LAMP_CHECK_LAUNCH();
    return launch_reduce_partials(part, S, O, dw, beta, s);
}
