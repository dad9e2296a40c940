// 1x1x1 head, softmax and cross entropy (forward and backward).  One thread per voxel; the
// op is bound by reading the activations and writing the fp32 logits.
#include "internal.h"
#include "vec.h"

namespace lamp {

static const int kMaxClasses = 16;

// KM: compile-time bound on the class count (4, 8 or 16).
// MODE 0: logits only.  MODE 1: + loss partials, dlogits, dx.
template <typename T, int VEC, int MODE, int KM>
__global__ __launch_bounds__(256) void head_kernel(const T* __restrict__ x, int ldx, NormIn nm, const T* __restrict__ wh,
                                                   const float* __restrict__ bh, int K, int C, int64_t Vs, int64_t Vtot,
                                                   const int32_t* __restrict__ labels, float* __restrict__ logits,
                                                   float* __restrict__ dlogits, T* __restrict__ dx, int lddx,
                                                   float* __restrict__ loss_part, float invV) {
    extern __shared__ float wsh[];  // [K][C]
    __shared__ float red[256];
    for (int i = threadIdx.x; i < K * C; i += 256) wsh[i] = io<T>::ld(wh + i);
    __syncthreads();
    float lsum = 0.f;
    for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < Vtot; v += (int64_t)gridDim.x * 256) {
        const int n = (int)(v / Vs);
        float acc[KM];
#pragma unroll
        for (int k = 0; k < KM; ++k) acc[k] = (k < K && bh) ? bh[k] : 0.f;
        const T* xp = x + v * ldx;
        for (int c0 = 0; c0 < C; c0 += VEC) {
            float xv[VEC];
            load_norm_vec<T, VEC>(xp + c0, nm, n, c0, xv);
#pragma unroll
            for (int i = 0; i < VEC; ++i)
#pragma unroll
                for (int k = 0; k < KM; ++k)
                    if (k < K) acc[k] = fmaf(xv[i], wsh[k * C + c0 + i], acc[k]);
        }
        if (logits) {
#pragma unroll
            for (int k = 0; k < KM; ++k)
                if (k < K) logits[v * K + k] = acc[k];
        }
        if (MODE == 1) {
            float m = acc[0];
#pragma unroll
            for (int k = 1; k < KM; ++k)
                if (k < K) m = acc[k] > m ? acc[k] : m;
            float se = 0.f;
#pragma unroll
            for (int k = 0; k < KM; ++k)
                if (k < K) se += expf(acc[k] - m);
            const float lse = m + logf(se);
            const int lab = labels[v];
            float ll = 0.f;
#pragma unroll
            for (int k = 0; k < KM; ++k) {
                if (k < K) {
                    if (k == lab) ll = acc[k];
                    float p = expf(acc[k] - lse);
                    acc[k] = (p - (k == lab ? 1.f : 0.f)) * invV;
                    dlogits[v * K + k] = acc[k];
                }
            }
            lsum += (lse - ll) * invV;
            if (dx) {
                for (int c0 = 0; c0 < C; c0 += VEC) {
                    float g[VEC];
#pragma unroll
                    for (int i = 0; i < VEC; ++i) {
                        g[i] = 0.f;
#pragma unroll
                        for (int k = 0; k < KM; ++k)
                            if (k < K) g[i] = fmaf(acc[k], wsh[k * C + c0 + i], g[i]);
                    }
                    Vec<T, VEC>::store(dx + v * lddx + c0, g);
                }
            }
        }
    }
    if (MODE == 1) {
        red[threadIdx.x] = lsum;
        __syncthreads();
        for (int off = 128; off > 0; off >>= 1) {
            if (threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
            __syncthreads();
        }
        if (threadIdx.x == 0) loss_part[blockIdx.x] = red[0];
    }
}

// part[s][k*C + c] = sum over the voxels of split s of dlogits[v][k] * X[v][c].  Threads side by
// side cover the channels of one voxel row (coalesced), 256/C voxel rows are in flight per block and
// every thread keeps K sums; the row lanes are then added in order through LDS.
template <typename T, int KM>
__global__ __launch_bounds__(256) void head_wgrad_kernel(const T* __restrict__ x, int ldx, NormIn nm,
                                                         const float* __restrict__ dlogits, int K, int C, int64_t Vs,
                                                         int64_t Vtot, int64_t vps, float* __restrict__ part) {
    __shared__ float red[KM * 256];
    const int cthreads = C < 256 ? C : 256;
    const int rl = 256 / cthreads;
    const int cl = threadIdx.x % cthreads, r0 = threadIdx.x / cthreads;
    const int c = blockIdx.y * 256 + cl;
    int64_t v0 = (int64_t)blockIdx.x * vps, v1 = v0 + vps;
    if (v1 > Vtot) v1 = Vtot;
    float acc[KM];
#pragma unroll
    for (int k = 0; k < KM; ++k) acc[k] = 0.f;
    if (r0 < rl && c < C)
        for (int64_t v = v0 + r0; v < v1; v += rl) {
            const float xv = load_norm(x + v * ldx + c, nm, (int)(v / Vs), c);
            const float* dl = dlogits + v * K;
#pragma unroll
            for (int k = 0; k < KM; ++k)
                if (k < K) acc[k] = fmaf(dl[k], xv, acc[k]);
        }
#pragma unroll
    for (int k = 0; k < KM; ++k)
        if (k < K) red[k * 256 + threadIdx.x] = acc[k];
    __syncthreads();
    if (r0 == 0 && c < C)
        for (int k = 0; k < K; ++k) {
            float t = 0.f;
            for (int r = 0; r < rl; ++r) t += red[k * 256 + r * cthreads + cl];
            part[(int64_t)blockIdx.x * K * C + (int64_t)k * C + c] = t;
        }
}

// ---- matrix-core head (bf16, C = 16 / 32 / 48 / 64 channels, up to 16 classes) ---------------------
// logits^T[class][voxel] = Wh[class][c] * x^T[c][voxel] with v_mfma_f32_32x32x16_bf16: the classes (padded
// to 32) are the rows, 32 voxels the columns, so the activations enter as 16 contiguous bytes per lane
// straight from global memory and every lane ends with 8 of its voxel's logits (classes 4*half + 0..3 and
// 8 + 4*half + 0..3; lane pair (l, l + 32) = one voxel).  Softmax and cross entropy take two exchanges
// inside the pair.  Backward in the same pass: dx^T[c][voxel] = Wh^T[c][class] * dlogits^T[class][voxel]
// (dlogits rounded to bf16 for this product), and dWh[class][c] += dlogits^T * x over the voxels with
// the fp32 instruction v_mfma_f32_32x32x2_f32, whose operands are one float per lane read from a
// [voxel][class] / [voxel][channel] staging tile in LDS; dbh from per-lane sums.  One pass over x.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 hbf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float hf32x16;

__device__ __forceinline__ uint32_t head_pack_bf16(float lo, float hi) { return (uint32_t)f2bf(lo) | ((uint32_t)f2bf(hi) << 16); }

// MODE 0: logits only.  MODE 1: + loss, dx, per-wave partials of dWh and dbh.
// NCB: 32-channel blocks the instantiation holds (C <= 32 * NCB).
// NORM: x is a raw conv output; InstanceNorm (+ ReLU) is applied while it is loaded, rounded to bf16 as the
// stored activation would be (every 32-voxel group lies inside one sample: Vs % 32 == 0).
// NI: classes a lane works on (4 serves up to 8 classes: 4*half + i; 8 serves 16).
template <int MODE, int NCB, bool NORM = false, int NI = 8>
__global__ __launch_bounds__(256, NCB == 1 ? 4 : NCB == 2 ? 3 : 1) void head_mfma_kernel(const bf16_t* __restrict__ x, int ldx, const bf16_t* __restrict__ wh,
                                                        const float* __restrict__ bh, int K, int C, int64_t Vtot,
                                                        const int32_t* __restrict__ labels, float* __restrict__ logits,
                                                        bf16_t* __restrict__ dx, int lddx, float* __restrict__ loss_part,
                                                        float* __restrict__ wpart, float* __restrict__ bpart, float invV,
                                                        NormIn nm = NormIn{nullptr, nullptr, nullptr, 0, 0}, int64_t Vs = 1) {
    __shared__ float dls[4][32][33];   // per wave: dlogits of 32 voxels x 32 (padded) classes
    __shared__ float xs[4][32][32 * NCB + 1];   // per wave: activations of 32 voxels x up to 32*NCB channels, fp32
    __shared__ float red[256];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, l32 = lane & 31, half = lane >> 5;
    const int CK = C >> 4;                 // 16-channel k-steps
    const int CB = (C + 31) >> 5;          // 32-channel row blocks of dx / column blocks of dWh
    // forward A fragments: row = class l32, k = channels 16*kc + 8*half + e
    hbf16x8 afw[2 * NCB], abw[NCB];
#pragma unroll
    for (int kc = 0; kc < 2 * NCB; ++kc) {
        uint4 q = make_uint4(0, 0, 0, 0);
        if (kc < CK && l32 < K) q = *reinterpret_cast<const uint4*>(wh + (size_t)l32 * C + 16 * kc + 8 * half);
        afw[kc] = __builtin_bit_cast(hbf16x8, q);
    }
    // backward A fragments: row = channel 32*cb + l32, k = classes 8*half + e
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
        uint32_t r[4] = {0, 0, 0, 0};
        const int ch = 32 * cb + l32;
        if (cb < CB && ch < C) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int k = 8 * half + e;
                const uint32_t b = k < K ? (uint32_t)wh[(size_t)k * C + ch] : 0u;
                r[e >> 1] |= b << (16 * (e & 1));
            }
        }
        abw[cb] = __builtin_bit_cast(hbf16x8, make_uint4(r[0], r[1], r[2], r[3]));
    }
    // this lane's 8 classes and their biases
    int cls[8];
    float bias[8];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        cls[i] = 8 * (i >> 2) + 4 * half + (i & 3);
        bias[i] = (bh && cls[i] < K) ? bh[cls[i]] : 0.f;
    }
    if (MODE == 1) {
        for (int i = lane; i < 32 * 33; i += 64) (&dls[wv][0][0])[i] = 0.f;   // classes 16..31 stay zero
    }
    hf32x16 accw[NCB];
    float dbsum[8];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) accw[cb][r] = 0.f;
#pragma unroll
    for (int i = 0; i < NI; ++i) dbsum[i] = 0.f;
    float lsum = 0.f;
    __shared__ __attribute__((aligned(16))) float nco[NORM ? 4 : 1][2][NORM ? 32 * NCB : 4];   // per wave: a[c], b[c] of its current sample
    int cur_n = -1;
    const int64_t groups = (Vtot + 31) / 32;
    // With normalise-on-load every wave walks a contiguous run of groups, so that the sample (and with it the
    // coefficients) changes at most a few times per wave; otherwise the groups are dealt round robin.
    const int64_t nwaves = (int64_t)gridDim.x * 4, wid = (int64_t)blockIdx.x * 4 + wv;
    const int64_t gpw = (groups + nwaves - 1) / nwaves;
    const int64_t g_lo = NORM ? wid * gpw : wid, g_hi = NORM ? (g_lo + gpw < groups ? g_lo + gpw : groups) : groups;
    const int64_t g_step = NORM ? 1 : nwaves;
    // the activations of a group are fetched one group ahead (not where that would spill: the backward
    // instantiation for 64 channels is at its register limit for three workgroups per CU)
    constexpr bool AHEAD = !(MODE == 1 && NCB == 2);
    uint4 xnext[AHEAD ? 2 * NCB : 1];
    auto fetch_x = [&](int64_t g, auto& q) __attribute__((always_inline)) {
        const int64_t v = g * 32 + l32;
        const bool ok = g < g_hi && v < Vtot;
        const bf16_t* xp = x + (ok ? v : 0) * ldx;
#pragma unroll
        for (int kc = 0; kc < 2 * NCB; ++kc) {
            q[kc] = make_uint4(0, 0, 0, 0);
            if (kc < CK && ok) q[kc] = *reinterpret_cast<const uint4*>(xp + 16 * kc + 8 * half);
        }
    };
    if constexpr (AHEAD) fetch_x(g_lo, xnext);
    for (int64_t g = g_lo; g < g_hi; g += g_step) {
        const int64_t v = g * 32 + l32;
        const bool valid = v < Vtot;
        if (NORM) {
            const int n = (int)((g * 32) / Vs);
            if (n != cur_n) {   // wave-uniform
                cur_n = n;
                __builtin_amdgcn_wave_barrier();
                for (int c = lane; c < C; c += 64) norm_coeffs(nm, n, c, nco[wv][0][c], nco[wv][1][c]);
                __builtin_amdgcn_wave_barrier();
            }
        }
        uint4 xq[2 * NCB];
        if constexpr (AHEAD) {
#pragma unroll
            for (int kc = 0; kc < 2 * NCB; ++kc) xq[kc] = xnext[kc];
            fetch_x(g + g_step, xnext);
        } else {
            fetch_x(g, xq);
        }
        hf32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
        for (int kc = 0; kc < 2 * NCB; ++kc) {
            if (kc < CK) {
                if (NORM) {
                    uint32_t r4[4] = {xq[kc].x, xq[kc].y, xq[kc].z, xq[kc].w};
                    float na[8], nb[8];
                    *reinterpret_cast<float4*>(na) = *reinterpret_cast<const float4*>(&nco[wv][0][16 * kc + 8 * half]);
                    *reinterpret_cast<float4*>(na + 4) = *reinterpret_cast<const float4*>(&nco[wv][0][16 * kc + 8 * half + 4]);
                    *reinterpret_cast<float4*>(nb) = *reinterpret_cast<const float4*>(&nco[wv][1][16 * kc + 8 * half]);
                    *reinterpret_cast<float4*>(nb + 4) = *reinterpret_cast<const float4*>(&nco[wv][1][16 * kc + 8 * half + 4]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float u0 = norm_u(__uint_as_float(r4[e] << 16), na[2 * e], nb[2 * e]);
                        float u1 = norm_u(__uint_as_float(r4[e] & 0xFFFF0000u), na[2 * e + 1], nb[2 * e + 1]);
                        if (nm.relu) { u0 = u0 > 0.f ? u0 : 0.f; u1 = u1 > 0.f ? u1 : 0.f; }
                        typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
                        typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
                        const f32x2 uu = {u0, u1};
                        r4[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(uu, bf16x2));   // round to nearest even
                    }
                    xq[kc] = valid ? make_uint4(r4[0], r4[1], r4[2], r4[3]) : make_uint4(0, 0, 0, 0);
                }
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afw[kc], __builtin_bit_cast(hbf16x8, xq[kc]), acc, 0, 0, 0);
            }
        }
        float lg[8];
#pragma unroll
        for (int i = 0; i < NI; ++i) lg[i] = acc[i] + bias[i];
        if (logits) {
            // the group's logits are 32*K consecutive floats: pack them in LDS ([voxel][class]) and store 16 bytes
            // per lane instead of eight 4-byte pieces per lane
            float* pk = &xs[wv][0][0];
            const int64_t left = Vtot - g * 32;   // valid voxels of the group (wave-uniform)
            if (left >= 32) {
#pragma unroll
                for (int i = 0; i < NI; ++i)
                    if (cls[i] < K) pk[l32 * K + cls[i]] = lg[i];
                __builtin_amdgcn_wave_barrier();
                float* dst = logits + g * 32 * K;
                for (int q4 = lane; q4 < 8 * K; q4 += 64)
                    *reinterpret_cast<float4*>(dst + 4 * q4) = *reinterpret_cast<const float4*>(pk + 4 * q4);
                __builtin_amdgcn_wave_barrier();
            } else if (valid) {
#pragma unroll
                for (int i = 0; i < NI; ++i)
                    if (cls[i] < K) logits[v * K + cls[i]] = lg[i];
            }
        }
        if (MODE == 1) {
            float m = -3.0e38f;
#pragma unroll
            for (int i = 0; i < NI; ++i)
                if (cls[i] < K) m = lg[i] > m ? lg[i] : m;
            const float mo = __shfl_xor(m, 32);
            m = mo > m ? mo : m;
            float se = 0.f, ex[8];
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                ex[i] = cls[i] < K ? expf(lg[i] - m) : 0.f;
                se += ex[i];
            }
            se += __shfl_xor(se, 32);
            const float lse = m + logf(se), rse = 1.0f / se;
            const int lab = valid ? labels[v] : -1;
            float ll = 0.f, dl[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                dl[i] = 0.f;
                if (cls[i] < K && valid) {
                    if (cls[i] == lab) ll = lg[i];
                    dl[i] = (ex[i] * rse - (cls[i] == lab ? 1.f : 0.f)) * invV;
                }
                dbsum[i] += dl[i];
            }
            ll += __shfl_xor(ll, 32);
            if (valid && half == 0) lsum += (lse - ll) * invV;
            // dlogits^T as the B operand of the dx product: this lane needs classes 8*half .. 8*half+7
            float snd[4], rcv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) snd[j] = half == 0 ? dl[4 + j] : dl[j];
#pragma unroll
            for (int j = 0; j < 4; ++j) rcv[j] = __shfl_xor(snd[j], 32);
            float bk[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                bk[j] = half == 0 ? dl[j] : rcv[j];
                bk[4 + j] = half == 0 ? rcv[j] : dl[4 + j];
            }
            const hbf16x8 bdl = __builtin_bit_cast(hbf16x8, make_uint4(head_pack_bf16(bk[0], bk[1]), head_pack_bf16(bk[2], bk[3]),
                                                                         head_pack_bf16(bk[4], bk[5]), head_pack_bf16(bk[6], bk[7])));
            if (dx) {
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb) {
                    if (cb < CB) {
                        hf32x16 a2;
#pragma unroll
                        for (int r = 0; r < 16; ++r) a2[r] = 0.f;
                        a2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(abw[cb], bdl, a2, 0, 0, 0);
                        // 32 voxels x 32 channels: through LDS (80-byte rows) so that four lanes store the 64 bytes of
                        // a voxel side by side
                        char* tp = reinterpret_cast<char*>(&xs[wv][0][0]);
#pragma unroll
                        for (int rg = 0; rg < 4; ++rg)
                            *reinterpret_cast<uint2*>(tp + l32 * 80 + (8 * rg + 4 * half) * 2) =
                                make_uint2(head_pack_bf16(a2[rg * 4 + 0], a2[rg * 4 + 1]), head_pack_bf16(a2[rg * 4 + 2], a2[rg * 4 + 3]));
                        __builtin_amdgcn_wave_barrier();
#pragma unroll
                        for (int it = 0; it < 2; ++it) {
                            const int vx = it * 16 + (lane >> 2), ch = 32 * cb + (lane & 3) * 8;
                            const uint4 q = *reinterpret_cast<const uint4*>(tp + vx * 80 + (lane & 3) * 16);
                            const int64_t vv = g * 32 + vx;
                            if (vv < Vtot && ch < C) *reinterpret_cast<uint4*>(dx + vv * lddx + ch) = q;
                        }
                        __builtin_amdgcn_wave_barrier();
                    }
                }
            }
            if (wpart) {
                // stage dlogits [voxel][class] and x [voxel][channel] (fp32) for the voxel-reduction product
#pragma unroll
                for (int i = 0; i < NI; ++i) dls[wv][l32][cls[i]] = dl[i];
#pragma unroll
                for (int kc = 0; kc < 2 * NCB; ++kc) {
                    if (kc < CK) {
                        const uint32_t r4[4] = {xq[kc].x, xq[kc].y, xq[kc].z, xq[kc].w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            xs[wv][l32][16 * kc + 8 * half + 2 * e] = __uint_as_float(r4[e] << 16);
                            xs[wv][l32][16 * kc + 8 * half + 2 * e + 1] = __uint_as_float(r4[e] & 0xFFFF0000u);
                        }
                    }
                }
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int kv = 0; kv < 16; ++kv) {
                    const float av = dls[wv][2 * kv + half][l32];
#pragma unroll
                    for (int cb = 0; cb < NCB; ++cb) {
                        if (cb < CB) {
                            const int ch = 32 * cb + l32;
                            const float bv = ch < C ? xs[wv][2 * kv + half][ch] : 0.f;
                            accw[cb] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, accw[cb], 0, 0, 0);
                        }
                    }
                }
                __builtin_amdgcn_wave_barrier();
            }
        }
    }
    if (MODE == 1) {
        red[threadIdx.x] = lsum;
        __syncthreads();
        for (int off = 128; off > 0; off >>= 1) {
            if (threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
            __syncthreads();
        }
        if (threadIdx.x == 0) loss_part[blockIdx.x] = red[0];
        const int slot = blockIdx.x * 4 + wv;
        if (wpart) {
            // accw: row = class 8*(r/4) + 4*half + (r%4), column = channel 32*cb + l32
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int k = 8 * (r >> 2) + 4 * half + (r & 3), ch = 32 * cb + l32;
                    if (cb < CB && k < K && ch < C) wpart[((size_t)slot * K + k) * C + ch] = accw[cb][r];
                }
        }
        if (bpart) {
            // fold the 32 voxel lanes of each half
#pragma unroll
            for (int i = 0; i < NI; ++i) {
#pragma unroll
                for (int m = 1; m < 32; m <<= 1) dbsum[i] += __shfl_xor(dbsum[i], m);
                if (l32 == 0 && cls[i] < K) bpart[(size_t)slot * K + cls[i]] = dbsum[i];
            }
        }
    }
}

static bool head_mfma_ok(const lamp_tensor_desc* xd, const void* x, const lamp_norm_in* xnorm, const void* wh, int classes,
                         const lamp_tensor_desc* dxd, const void* dx, const void* logits, bool allow_norm = false) {
    bool nm = xnorm && xnorm->mean_rstd && xnorm->c_norm > 0;
    // normalise-on-load: forward only, all channels, voxel groups that do not straddle samples
    if (nm && allow_norm && xnorm->c_norm == xd->c && ((int64_t)xd->d * xd->h * xd->w) % 32 == 0) nm = false;
    if (xd->dtype != LAMP_BF16 || nm || xd->c % 16 || xd->c > 128 || xd->ldc % 8 || classes > 16) return false;
    if (!aligned16(x) || !aligned16(wh)) return false;
    if (dx && (dxd->ldc % 8 || !aligned16(dx))) return false;
    if (logits && !aligned16(logits)) return false;
    return true;
}
// Workgroups of the matrix-core head: every one walks the same number of voxel groups, so the grid is at most
// what is resident at once (`per_cu` workgroups on each of the 256 CUs); a partial second round would leave
// most of the chip idle for half of the run.  4 * blocks <= 4096 partial slots.
static int head_mfma_blocks(int64_t V, int per_cu = 4) {
    int64_t b = ((V + 31) / 32 + 3) / 4;
    const int64_t cap = 256 * (int64_t)per_cu;
    return (int)(b > cap ? cap : (b < 1 ? 1 : b));
}

static int head_blocks(int64_t V) {
    int64_t b = (V + 255) / 256;
    return (int)(b > 2048 ? 2048 : b);
}
static int head_splits(int64_t V) {
    int64_t s = (V + 511) / 512;
    return (int)(s > 4096 ? 4096 : (s < 1 ? 1 : s));
}
static int head_mfma_blocks(int64_t V, int per_cu);
// partial slots of the weight gradient the workspace must hold: the generic path's splits or one per wave
// of the matrix-core path
static int head_wslots(int64_t V) {
    const int a = head_splits(V), b = 4 * head_mfma_blocks(V);
    return a > b ? a : b;
}

static lamp_status head_check(const lamp_tensor_desc* xd, const void* x, const void* wh, int classes) {
    if (!xd || !x || !wh) return LAMP_ERR_NULL;
    if (!desc_ok(xd) || classes < 1 || classes > kMaxClasses) return LAMP_ERR_SHAPE;
    if ((size_t)classes * xd->c * sizeof(float) > 48 * 1024) return LAMP_ERR_UNSUPPORTED;
    return LAMP_OK;
}

}  // namespace lamp

using namespace lamp;

#define LAMP_DISPATCH_KM(k, BODY)                      \
    do {                                               \
        if ((k) <= 4) { constexpr int KM = 4; BODY }   \
        else if ((k) <= 8) { constexpr int KM = 8; BODY } \
        else { constexpr int KM = 16; BODY }           \
    } while (0)

extern "C" lamp_status lamp_head_fwd(const lamp_tensor_desc* xd, const void* x, const lamp_norm_in* xnorm, const void* wh,
                                     const float* bh, int classes, float* logits, void* stream) {
    lamp_status st = head_check(xd, x, wh, classes);
    if (st != LAMP_OK) return st;
    if (!logits) return LAMP_ERR_NULL;
    if ((st = norm_ok(xnorm, xd)) != LAMP_OK) return st;
    const int64_t Vs = (int64_t)xd->d * xd->h * xd->w, Vt = nvox(xd);
    if (head_mfma_ok(xd, x, xnorm, wh, classes, nullptr, nullptr, logits, true)) {
        if (xnorm && xnorm->mean_rstd && xnorm->c_norm > 0) {
            const NormIn nm = make_norm(xnorm);
            if (xd->c <= 64)
                hipLaunchKernelGGL((head_mfma_kernel<0, 2, true>), dim3(head_mfma_blocks(Vt)), dim3(256), 0, (hipStream_t)stream,
                                   (const bf16_t*)x, xd->ldc, (const bf16_t*)wh, bh, classes, xd->c, Vt, nullptr, logits, nullptr,
                                   0, nullptr, nullptr, nullptr, 0.f, nm, Vs);
            else
                hipLaunchKernelGGL((head_mfma_kernel<0, 4, true>), dim3(head_mfma_blocks(Vt)), dim3(256), 0, (hipStream_t)stream,
                                   (const bf16_t*)x, xd->ldc, (const bf16_t*)wh, bh, classes, xd->c, Vt, nullptr, logits, nullptr,
                                   0, nullptr, nullptr, nullptr, 0.f, nm, Vs);
            LAMP_CHECK_LAUNCH();
            return LAMP_OK;
        }
        if (xd->c <= 64)
            hipLaunchKernelGGL((head_mfma_kernel<0, 2>), dim3(head_mfma_blocks(Vt)), dim3(256), 0, (hipStream_t)stream,
                               (const bf16_t*)x, xd->ldc, (const bf16_t*)wh, bh, classes, xd->c, Vt, nullptr, logits, nullptr, 0,
                               nullptr, nullptr, nullptr, 0.f);
        else
            hipLaunchKernelGGL((head_mfma_kernel<0, 4>), dim3(head_mfma_blocks(Vt)), dim3(256), 0, (hipStream_t)stream,
                               (const bf16_t*)x, xd->ldc, (const bf16_t*)wh, bh, classes, xd->c, Vt, nullptr, logits, nullptr, 0,
                               nullptr, nullptr, nullptr, 0.f);
        LAMP_CHECK_LAUNCH();
        return LAMP_OK;
    }
    const size_t shm = (size_t)classes * xd->c * sizeof(float);
    NormIn nm = make_norm(xnorm);
    const int vec = pick_vec(xd->dtype, xd->c, {xd->ldc}, {x});
    LAMP_DISPATCH_TV(xd->dtype, vec, {
        LAMP_DISPATCH_KM(classes, {
            hipLaunchKernelGGL((head_kernel<T, VEC, 0, KM>), dim3(head_blocks(Vt)), dim3(256), shm, (hipStream_t)stream,
                               (const T*)x, xd->ldc, nm, (const T*)wh, bh, classes, xd->c, Vs, Vt, nullptr, logits,
                               nullptr, (T*)nullptr, 0, nullptr, 0.f);
        });
    });
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}

extern "C" size_t lamp_head_ce_workspace_bytes(const lamp_tensor_desc* xd, int classes) {
    if (!desc_ok(xd) || classes < 1) return 0;
    const int64_t Vt = nvox(xd);
    return align_up((size_t)Vt * classes * sizeof(float)) + align_up((size_t)2048 * sizeof(float)) +
           align_up((size_t)head_wslots(Vt) * classes * xd->c * sizeof(float)) + colsum_ws_bytes(Vt, classes) +
           align_up((size_t)4096 * classes * sizeof(float));
}

extern "C" lamp_status lamp_head_ce(const lamp_tensor_desc* xd, const void* x, const lamp_norm_in* xnorm, const void* wh,
                                    const float* bh, int classes, const int32_t* labels, float* logits, float* loss,
                                    const lamp_tensor_desc* dxd, void* dx, float* dwh, float* dbh, float beta, void* ws,
                                    size_t ws_bytes, void* stream) {
    return lamp::head_ce_run(xd, x, xnorm, wh, bh, classes, labels, logits, loss, dxd, dx, dwh, dbh, beta, 0, 0.f, ws, ws_bytes,
                             stream);
}

// norm_count: the voxel count the mean is taken over (0: this call's own voxels); a micro-batch of a
// larger mini-batch passes the mini-batch's count, so that losses and gradients of the micro-batches
// add up to the mini-batch's.  loss_beta: 1 adds this call's loss to *loss instead of overwriting it.
lamp_status lamp::head_ce_run(const lamp_tensor_desc* xd, const void* x, const lamp_norm_in* xnorm, const void* wh,
                              const float* bh, int classes, const int32_t* labels, float* logits, float* loss,
                              const lamp_tensor_desc* dxd, void* dx, float* dwh, float* dbh, float beta, int64_t norm_count,
                              float loss_beta, void* ws, size_t ws_bytes, void* stream) {
    lamp_status st = head_check(xd, x, wh, classes);
    if (st != LAMP_OK) return st;
    if (!labels || !loss) return LAMP_ERR_NULL;
    if ((st = norm_ok(xnorm, xd)) != LAMP_OK) return st;
    if (beta != 0.f && beta != 1.f) return LAMP_ERR_SHAPE;
    int lddx = 0;
    if (dx) {
        if (!dxd) return LAMP_ERR_NULL;
        if (!desc_ok(dxd) || !same_space(xd, dxd) || dxd->c != xd->c) return LAMP_ERR_SHAPE;
        if (dxd->dtype != xd->dtype) return LAMP_ERR_DTYPE;
        lddx = dxd->ldc;
    }
    if (!ws || ws_bytes < lamp_head_ce_workspace_bytes(xd, classes)) return LAMP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int64_t Vs = (int64_t)xd->d * xd->h * xd->w, Vt = nvox(xd);
    const float invV = 1.0f / (float)(norm_count > 0 ? norm_count : Vt);
    const int K = classes, C = xd->c;
    Carver cv(ws, ws_bytes);
    float* dlogits = (float*)cv.take((size_t)Vt * K * sizeof(float));
    const int nb = head_blocks(Vt);
    float* lpart = (float*)cv.take((size_t)2048 * sizeof(float));   // one loss partial per workgroup of either path
    const int S = head_splits(Vt);
    float* wpart = (float*)cv.take((size_t)head_wslots(Vt) * K * C * sizeof(float));
    const size_t csb = colsum_ws_bytes(Vt, K);
    void* csws = cv.take(csb);
    if (!cv.ok()) return LAMP_ERR_WORKSPACE;
    if (head_mfma_ok(xd, x, xnorm, wh, K, dxd, dx, logits)) {
        // one pass: logits, loss, dx, per-wave partials of dWh and dbh (the dlogits buffer is not used)
        float* bpart = (float*)cv.take((size_t)4096 * K * sizeof(float));
        if (!cv.ok()) return LAMP_ERR_WORKSPACE;
        const int nbm = head_mfma_blocks(Vt, C <= 32 ? 4 : C <= 64 ? 3 : 4);   // 4 * nbm <= 4096 partial slots
#define LAMP_HEAD_BWD(NCB_, NI_)                                                                                                   \
    hipLaunchKernelGGL((head_mfma_kernel<1, NCB_, false, NI_>), dim3(nbm), dim3(256), 0, s, (const bf16_t*)x, xd->ldc, (const bf16_t*)wh, \
                       bh, K, C, Vt, labels, logits, (bf16_t*)dx, lddx, lpart, dwh ? wpart : nullptr, dbh ? bpart : nullptr, invV)
        if (K <= 8) {   // the usual few classes: half the per-class work of a lane
            if (C <= 32) LAMP_HEAD_BWD(1, 4);
            else if (C <= 64) LAMP_HEAD_BWD(2, 4);
            else LAMP_HEAD_BWD(4, 4);
        } else {
            if (C <= 32) LAMP_HEAD_BWD(1, 8);
            else if (C <= 64) LAMP_HEAD_BWD(2, 8);
            else LAMP_HEAD_BWD(4, 8);
        }
#undef LAMP_HEAD_BWD
        LAMP_CHECK_LAUNCH();
        if ((st = launch_reduce_partials(lpart, nbm, 1, loss, loss_beta, s)) != LAMP_OK) return st;
        if (dwh && (st = launch_reduce_partials(wpart, nbm * 4, (int64_t)K * C, dwh, beta, s)) != LAMP_OK) return st;
        if (dbh && (st = launch_reduce_partials(bpart, nbm * 4, K, dbh, beta, s)) != LAMP_OK) return st;
        return LAMP_OK;
    }
    const size_t shm = (size_t)K * C * sizeof(float);
    NormIn nm = make_norm(xnorm);
    const int vec = pick_vec(xd->dtype, C, {xd->ldc, lddx}, {x, dx});
    LAMP_DISPATCH_TV(xd->dtype, vec, {
        LAMP_DISPATCH_KM(K, {
            hipLaunchKernelGGL((head_kernel<T, VEC, 1, KM>), dim3(nb), dim3(256), shm, s, (const T*)x, xd->ldc, nm,
                               (const T*)wh, bh, K, C, Vs, Vt, labels, logits, dlogits, (T*)dx, lddx, lpart, invV);
        });
    });
    LAMP_CHECK_LAUNCH();
    if ((st = launch_reduce_partials(lpart, nb, 1, loss, loss_beta, s)) != LAMP_OK) return st;
    if (dwh) {
        const int64_t vps = (Vt + S - 1) / S;
        dim3 grid(S, cdiv(C, 256));
        LAMP_DISPATCH_KM(K, {
            if (xd->dtype == LAMP_BF16)
                hipLaunchKernelGGL((head_wgrad_kernel<bf16_t, KM>), grid, dim3(256), 0, s, (const bf16_t*)x, xd->ldc, nm,
                                   dlogits, K, C, Vs, Vt, vps, wpart);
            else
                hipLaunchKernelGGL((head_wgrad_kernel<float, KM>), grid, dim3(256), 0, s, (const float*)x, xd->ldc, nm,
                                   dlogits, K, C, Vs, Vt, vps, wpart);
        });
        LAMP_CHECK_LAUNCH();
        if ((st = launch_reduce_partials(wpart, S, (int64_t)K * C, dwh, beta, s)) != LAMP_OK) return st;
    }
    if (dbh) {
        if ((st = launch_colsum(dlogits, LAMP_F32, Vt, K, K, dbh, beta, csws, csb, s)) != LAMP_OK) return st;
    }
    return LAMP_OK;
}
