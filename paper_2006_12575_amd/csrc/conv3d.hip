// 3x3x3 convolution: public entry points, argument checking, kernel selection, and the generic
// direct kernels (any dtype / channel count) that serve the fp32 path and odd channel counts.
// Shapes with channel counts in multiples of 32 in bf16 go to the matrix-core kernels.
#include "internal.h"
#include "vec.h"

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

// Forward for Cin == 1 with C_out = 32*CB on the matrix cores: z^T[co][voxel] = W[co][tap] * X27^T[tap][voxel],
// taps (27, padded to 32) as the reduction dimension, weights kept in registers as the A operand.
// A workgroup walks blocks of four output rows (one per wave) of one sample: the 3 x 6 input rows a
// block needs are staged in LDS (zero padded), and the B operand -- the 27 neighbours of 32 voxels
// -- is gathered from there with 16-bit LDS reads.  The weight rows are permuted so that a lane ends
// with 16 consecutive channels of its voxel; a per-wave LDS transpose turns that into whole 64-byte
// pieces for the store (four lanes side by side), and the per-channel sum / sum of squares of the
// rounded outputs are accumulated on the way for the instance-norm statistics.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 c1_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float c1_f32x16;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float c1_f32x2;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 c1_bf16x2;
__device__ __forceinline__ uint32_t c1_pack(float lo, float hi) {
    c1_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, c1_bf16x2));
}

struct Cin1Args {
    const bf16_t* x; int ldx;
    const bf16_t* w;
    bf16_t* z; int ldz;
    int N, D, H, W;
    int G;           // 32-voxel groups per row
    int WP, RS;      // staged row: WP = 32*G + 2 elements (w = -1 .. 32*G), row stride RS elements
    uint32_t mWP; int sWP;   // e / WP == (e * mWP) >> sWP for e < 2^31
    float* partial;  // [N][parts][C][2] per-wave (sum, sum of squares), or nullptr
    int32_t* counts; // [N][parts] voxels behind each partial
};

static constexpr int C1_TROW = 80;  // bytes per voxel row of the transposing buffer (64 of data, padded)

template <int CB, int NE>
__global__ __launch_bounds__(256) void conv3d_cin1_fwd_tile_kernel(Cin1Args a) {
    extern __shared__ __attribute__((aligned(16))) char c1_lds[];
    char* tb = c1_lds + threadIdx.x / 64 * (32 * C1_TROW);          // this wave's transposing buffer
    unsigned short* xt = reinterpret_cast<unsigned short*>(c1_lds + 4 * 32 * C1_TROW);  // [18][RS]
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, half = lane >> 5;
    const int n = blockIdx.y;
    const int C = 32 * CB;

    // A operand: MFMA row rho of block cb carries channel 32*cb + 16*((rho>>2)&1) + 4*(rho>>3) + (rho&3), so
    // that a lane's 16 accumulator registers are channels 32*cb + 16*half + 0..15 of its voxel
    c1_bf16x8 wa[CB][2];
    {
        const int ch = 16 * ((l32 >> 2) & 1) + 4 * (l32 >> 3) + (l32 & 3);
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                uint32_t r[4] = {0, 0, 0, 0};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int t = 16 * kb + 8 * half + e;
                    const uint32_t b = t < 27 ? (uint32_t)a.w[(size_t)(32 * cb + ch) * 27 + t] : 0u;
                    r[e >> 1] |= b << (16 * (e & 1));
                }
                wa[cb][kb] = __builtin_bit_cast(c1_bf16x8, make_uint4(r[0], r[1], r[2], r[3]));
            }
    }
    // B operand: element offsets of the lane's 16 taps inside the staged rows (padded taps repeat tap 26;
    // their weights are zero)
    int toff[2][8];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int t = 16 * kb + 8 * half + e;
            if (t > 26) t = 26;
            const int kd = t / 9, kh = (t / 3) % 3, kw = t % 3;
            toff[kb][e] = (kd * 6 + kh + wv) * a.RS + kw + l32;
        }

    float csum[CB][8], csq[CB][8];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int e = 0; e < 8; ++e) { csum[cb][e] = 0.f; csq[cb][e] = 0.f; }
    int32_t count = 0;

    const int hblocks = (a.H + 3) >> 2;
    const int nblk = a.D * hblocks;
    const int total_e = 18 * a.WP;
    const bf16_t* xs = a.x + (int64_t)n * a.D * a.H * a.W * a.ldx;
    for (int blk = blockIdx.x; blk < nblk; blk += gridDim.x) {
        const int d = blk / hblocks, h0 = (blk - d * hblocks) << 2;
        // stage rows (kd, hh): input plane d + kd - 1, input row h0 - 1 + hh, columns w = -1 .. 32*G
        unsigned short stg[NE];
#pragma unroll
        for (int i = 0; i < NE; ++i) {
            const int e = tid + 256 * i;
            const int r = (int)(((uint64_t)(uint32_t)e * a.mWP) >> a.sWP), j = e - r * a.WP;
            const int kd = r / 6, hh = r - kd * 6;
            const int id = d + kd - 1, ih = h0 - 1 + hh, iw = j - 1;
            const bool in = e < total_e && id >= 0 && id < a.D && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
            stg[i] = in ? xs[(((int64_t)id * a.H + ih) * a.W + iw) * a.ldx] : (unsigned short)0;
        }
        __syncthreads();  // every wave is done with the previous block's rows
#pragma unroll
        for (int i = 0; i < NE; ++i) {
            const int e = tid + 256 * i;
            const int r = (int)(((uint64_t)(uint32_t)e * a.mWP) >> a.sWP), j = e - r * a.WP;
            if (e < total_e) xt[r * a.RS + j] = stg[i];
        }
        __syncthreads();
        const int h = h0 + wv;
        if (h < a.H) {
            bf16_t* zrow = a.z + ((((int64_t)n * a.D + d) * a.H + h) * a.W) * a.ldz;
            for (int g = 0; g < a.G; ++g) {
                c1_bf16x8 b[2];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    uint32_t r[4];
#pragma unroll
                    for (int e2 = 0; e2 < 4; ++e2) {
                        const uint32_t lo = xt[toff[kb][2 * e2] + 32 * g], hi = xt[toff[kb][2 * e2 + 1] + 32 * g];
                        r[e2] = lo | (hi << 16);
                    }
                    b[kb] = __builtin_bit_cast(c1_bf16x8, make_uint4(r[0], r[1], r[2], r[3]));
                }
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    c1_f32x16 acc;
#pragma unroll
                    for (int q = 0; q < 16; ++q) acc[q] = 0.f;
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa[cb][0], b[0], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa[cb][1], b[1], acc, 0, 0, 0);
#pragma unroll
                    for (int q4 = 0; q4 < 2; ++q4) {
                        const uint4 pk = make_uint4(c1_pack(acc[8 * q4 + 0], acc[8 * q4 + 1]), c1_pack(acc[8 * q4 + 2], acc[8 * q4 + 3]),
                                                    c1_pack(acc[8 * q4 + 4], acc[8 * q4 + 5]), c1_pack(acc[8 * q4 + 6], acc[8 * q4 + 7]));
                        *reinterpret_cast<uint4*>(tb + l32 * C1_TROW + half * 32 + q4 * 16) = pk;
                    }
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int it = 0; it < 2; ++it) {
                        const int vx = it * 16 + (lane >> 2), wq = 32 * g + vx;
                        const uint4 q = *reinterpret_cast<const uint4*>(tb + vx * C1_TROW + (lane & 3) * 16);
                        if (wq < a.W) {
                            *reinterpret_cast<uint4*>(zrow + (int64_t)wq * a.ldz + 32 * cb + (lane & 3) * 8) = q;
                            const uint32_t r4[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float f0 = __uint_as_float(r4[e] << 16), f1 = __uint_as_float(r4[e] & 0xFFFF0000u);
                                csum[cb][2 * e] += f0; csq[cb][2 * e] = fmaf(f0, f0, csq[cb][2 * e]);
                                csum[cb][2 * e + 1] += f1; csq[cb][2 * e + 1] = fmaf(f1, f1, csq[cb][2 * e + 1]);
                            }
                        }
                    }
                    __builtin_amdgcn_wave_barrier();
                }
            }
            count += a.W;
        }
    }
    if (a.partial) {
        // lanes with equal (lane & 3) hold the same 8 channels of different voxels
        const int part = blockIdx.x * 4 + wv, parts = gridDim.x * 4;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float sv = csum[cb][e], qv = csq[cb][e];
#pragma unroll
                for (int m = 4; m < 64; m <<= 1) { sv += __shfl_xor(sv, m); qv += __shfl_xor(qv, m); }
                if (lane < 4) {
                    const size_t o = (((size_t)n * parts + part) * C + 32 * cb + lane * 8 + e) * 2;
                    a.partial[o] = sv;
                    a.partial[o + 1] = qv;
                }
            }
        if (lane == 0) a.counts[(size_t)n * parts + part] = count;
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
    // four groups per round: all 64 two-byte loads of a round are in flight before its first multiply
    // (the voxel count is below 2^31: 32-bit index arithmetic)
    for (int64_t gb = g0; gb < g1; gb += 4) {
        U16x8 a[4], b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t g = gb + u;
            const bool live = g < g1;
            const uint32_t v = (uint32_t)((live ? g : g0) * 16 + 8 * kg);  // the lane's 8 voxels v..v+7 lie in one W-row
            const uint32_t w0 = v % (uint32_t)W;
            uint32_t r = v / (uint32_t)W;
            const int h = (int)(r % (uint32_t)H);
            r /= (uint32_t)H;
            const int d = (int)(r % (uint32_t)D);
            const int n = (int)(r / (uint32_t)D);
            const bf16_t* dp = dz + (int64_t)v * lddz + cob + l32;
#pragma unroll
            for (int e = 0; e < 8; ++e) a[u].e[e] = live ? dp[(int64_t)e * lddz] : (bf16_t)0;
            const int id = d + kd, ih = h + kh;
            const bool rowok = live && tap < 27 && id >= 0 && id < D && ih >= 0 && ih < H;
            const int64_t base = rowok ? (((int64_t)n * D + id) * H + ih) * W : 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int iw = (int)w0 + e + kw;
                const bool ok = rowok && iw >= 0 && iw < W;
                b[u].e[e] = ok ? x[(base + iw) * ldx] : (bf16_t)0;
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[u]), __builtin_bit_cast(bf16x8, b[u]), acc, 0,
                                                          0, 0);
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

// Weight gradient for Cin == 1 with the operands staged in LDS (C_out = 32*CB per workgroup column):
// dW[co][tap] = sum_v dz[v][co] * x[v + tap], voxels as the reduction dimension.  A workgroup walks
// blocks of four output rows (one per wave) like the tiled forward kernel and stages the 3 x 6 input
// rows the same way.  Per 16 voxels of its row a wave fetches dz with one 16-byte load per lane and
// 32 channels (two groups ahead), passes it through a private LDS slot and reads the A operand
// (dz^T, voxel-major per lane) with the transposing LDS load; the B operand -- 8 consecutive voxels
// shifted by the lane's tap -- is 8 two-byte LDS reads at immediate offsets.  Every wave writes its
// own partial [C_out][27] slab.
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short c1_s16x4;
__device__ __forceinline__ c1_bf16x8 c1_frag_tr(const char* p) {
    typedef __attribute__((address_space(3))) c1_s16x4 lds_s16x4;
    c1_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
    c1_s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 256));
    typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(c1_bf16x8, v);
}

struct Cin1WArgs {
    const bf16_t* x; int ldx;
    const bf16_t* dz; int lddz;
    float* part;     // [waves][Co][27]
    int N, D, H, W, Co;
    int G;           // 16-voxel groups per row
    int WP, RS;      // staged row: WP = 16*G + 2 elements (w = -1 .. 16*G), row stride RS elements
    uint32_t mWP; int sWP;
};

template <int CB, int NE>
__global__ __launch_bounds__(256) void conv3d_cin1_wgrad_tile_kernel(Cin1WArgs a) {
    extern __shared__ __attribute__((aligned(16))) char c1w_lds[];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, half = lane >> 5;
    char* slot = c1w_lds + wv * (2 * CB * 1024);                                         // two dz buffers of this wave
    unsigned short* xt = reinterpret_cast<unsigned short*>(c1w_lds + 4 * 2 * CB * 1024);  // [18][RS]
    const int co0 = blockIdx.y * (32 * CB);
    const int tap = l32 < 27 ? l32 : 26;   // columns 27..31 repeat tap 26 and are not written
    const int kd = tap / 9, kh = (tap / 3) % 3, kw = tap % 3;
    const int xoff = (kd * 6 + kh + wv) * a.RS + kw + 8 * half;
    // lane part of a transposing fragment read: voxel row 8*(b/2) + s/4, channel bytes 32*(b%2) + 8*(s%4)
    const int b16 = lane >> 4, s16 = lane & 15;
    const uint32_t loff = (uint32_t)((8 * (b16 >> 1) + (s16 >> 2)) * 64 + 32 * (b16 & 1) + 8 * (s16 & 3));
    const int vx = lane >> 2, piece = lane & 3;   // dz copy: voxel of the group, 16-byte piece of its 64 bytes

    c1_f32x16 acc[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[cb][r] = 0.f;

    const int hblocks = (a.H + 3) >> 2;
    const int per_n = a.D * hblocks;
    const int nblk = a.N * per_n;
    const int total_e = 18 * a.WP;
    for (int blk = blockIdx.x; blk < nblk; blk += gridDim.x) {
        const int n = blk / per_n, rblk = blk - n * per_n;
        const int d = rblk / hblocks, h0 = (rblk - d * hblocks) << 2;
        const bf16_t* xs = a.x + (int64_t)n * a.D * a.H * a.W * a.ldx;
        unsigned short stg[NE];
#pragma unroll
        for (int i = 0; i < NE; ++i) {
            const int e = tid + 256 * i;
            const int r = (int)(((uint64_t)(uint32_t)e * a.mWP) >> a.sWP), j = e - r * a.WP;
            const int skd = r / 6, hh = r - skd * 6;
            const int id = d + skd - 1, ih = h0 - 1 + hh, iw = j - 1;
            const bool in = e < total_e && id >= 0 && id < a.D && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
            stg[i] = in ? xs[(((int64_t)id * a.H + ih) * a.W + iw) * a.ldx] : (unsigned short)0;
        }
        __syncthreads();  // every wave is done with the previous block's rows
#pragma unroll
        for (int i = 0; i < NE; ++i) {
            const int e = tid + 256 * i;
            const int r = (int)(((uint64_t)(uint32_t)e * a.mWP) >> a.sWP), j = e - r * a.WP;
            if (e < total_e) xt[r * a.RS + j] = stg[i];
        }
        __syncthreads();
        const int h = h0 + wv;
        if (h < a.H) {
            const bf16_t* dzrow = a.dz + ((((int64_t)n * a.D + d) * a.H + h) * a.W) * a.lddz + co0 + piece * 8;
            auto fetch = [&](int g, uint4 (&q)[CB]) {
                const int w = 16 * g + vx;
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    q[cb] = make_uint4(0, 0, 0, 0);
                    if (g < a.G && w < a.W) q[cb] = *reinterpret_cast<const uint4*>(dzrow + (int64_t)w * a.lddz + 32 * cb);
                }
            };
            uint4 q0[CB], q1[CB];
            fetch(0, q0);
            fetch(1, q1);
            for (int g = 0; g < a.G; ++g) {
                char* buf = slot + (g & 1) * (CB * 1024);
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) *reinterpret_cast<uint4*>(buf + cb * 1024 + vx * 64 + piece * 16) = q0[cb];
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) q0[cb] = q1[cb];
                fetch(g + 2, q1);
                __builtin_amdgcn_wave_barrier();
                uint32_t r[4];
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const uint32_t lo = xt[xoff + 16 * g + 2 * e2], hi = xt[xoff + 16 * g + 2 * e2 + 1];
                    r[e2] = lo | (hi << 16);
                }
                const c1_bf16x8 b = __builtin_bit_cast(c1_bf16x8, make_uint4(r[0], r[1], r[2], r[3]));
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
                    acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(c1_frag_tr(buf + cb * 1024 + loff), b, acc[cb], 0, 0, 0);
            }
        }
    }
    if (l32 < 27) {
        float* pb = a.part + ((int64_t)blockIdx.x * 4 + wv) * a.Co * 27;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int co = co0 + 32 * cb + 8 * (r / 4) + 4 * half + (r % 4);
                pb[(int64_t)co * 27 + l32] = acc[cb][r];
            }
    }
}

static bool cin1_fwd_ok(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd, const lamp_norm_in* xnorm, const float* bias,
                        const void* z) {
    const bool nm = xnorm && xnorm->mean_rstd && xnorm->c_norm > 0;
    return xd->dtype == LAMP_BF16 && xd->c == 1 && !nm && !bias && zd->c % 8 == 0 && zd->c <= 128 && zd->ldc % 8 == 0 &&
           aligned16(z);
}
// ---- tiled Cin == 1 forward: launch geometry, workspace, dispatch ----
static int cin1_tile_groups(const lamp_tensor_desc* zd) { return (zd->w + 31) / 32; }
static int cin1_tile_ne(const lamp_tensor_desc* zd) { return (18 * (32 * cin1_tile_groups(zd) + 2) + 255) / 256; }
static bool cin1_tile_ok(const lamp_tensor_desc* zd) {
    return (zd->c == 32 || zd->c == 64 || zd->c == 128) && cin1_tile_ne(zd) <= 40 && zd->n <= 65535 &&
           (int64_t)zd->d * ((zd->h + 3) / 4) < ((int64_t)1 << 31);
}
static int cin1_tile_gridx(const lamp_tensor_desc* zd) {
    const int64_t nblk = (int64_t)zd->d * ((zd->h + 3) / 4);
    int64_t g = 2048 / zd->n;
    if (g < 1) g = 1;
    return (int)(nblk < g ? nblk : g);
}
static size_t cin1_tile_ws_bytes(const lamp_tensor_desc* zd) {
    const size_t parts = (size_t)cin1_tile_gridx(zd) * 4;
    return align_up((size_t)zd->n * parts * zd->c * 2 * sizeof(float)) + align_up((size_t)zd->n * parts * sizeof(int32_t));
}
template <int CB>
static void cin1_tile_launch(int ne, dim3 grid, size_t lds, hipStream_t s, const Cin1Args& a) {
    if (ne <= 12) hipLaunchKernelGGL((conv3d_cin1_fwd_tile_kernel<CB, 12>), grid, dim3(256), lds, s, a);
    else if (ne <= 20) hipLaunchKernelGGL((conv3d_cin1_fwd_tile_kernel<CB, 20>), grid, dim3(256), lds, s, a);
    else hipLaunchKernelGGL((conv3d_cin1_fwd_tile_kernel<CB, 40>), grid, dim3(256), lds, s, a);
}
static lamp_status cin1_tile_fwd(const lamp_tensor_desc* xd, const void* x, const void* w, const lamp_tensor_desc* zd, void* z,
                                 float* stats_out, float eps, void* ws, size_t ws_bytes, hipStream_t s) {
    Cin1Args a;
    a.x = (const bf16_t*)x; a.ldx = xd->ldc; a.w = (const bf16_t*)w; a.z = (bf16_t*)z; a.ldz = zd->ldc;
    a.N = zd->n; a.D = zd->d; a.H = zd->h; a.W = zd->w;
    a.G = cin1_tile_groups(zd);
    a.WP = 32 * a.G + 2;
    a.RS = a.WP;
    {   // round-up reciprocal: e / WP == (e * m) >> sh for e < 2^31
        int l = 0;
        while ((1 << l) < a.WP) ++l;
        a.sWP = 31 + l;
        a.mWP = (uint32_t)((((uint64_t)1 << (31 + l)) + (uint64_t)a.WP - 1) / (uint64_t)a.WP);
    }
    const int gx = cin1_tile_gridx(zd);
    const int parts = gx * 4;
    a.partial = nullptr; a.counts = nullptr;
    if (stats_out) {
        if (!ws || ws_bytes < cin1_tile_ws_bytes(zd)) return LAMP_ERR_WORKSPACE;
        a.partial = (float*)ws;
        a.counts = (int32_t*)((char*)ws + align_up((size_t)zd->n * parts * zd->c * 2 * sizeof(float)));
    }
    const size_t lds = 4 * 32 * C1_TROW + (size_t)18 * a.RS * sizeof(unsigned short);
    const dim3 grid(gx, zd->n);
    const int ne = cin1_tile_ne(zd);
    if (zd->c == 32) cin1_tile_launch<1>(ne, grid, lds, s, a);
    else if (zd->c == 64) cin1_tile_launch<2>(ne, grid, lds, s, a);
    else cin1_tile_launch<4>(ne, grid, lds, s, a);
    LAMP_CHECK_LAUNCH();
    if (stats_out) return launch_stats_finalize(a.partial, a.counts, parts, zd->n, zd->c, eps, stats_out, s, true);
    return LAMP_OK;
}
// ---- tiled Cin == 1 weight gradient: launch geometry, workspace, dispatch ----
static int cin1_wtile_groups(const lamp_tensor_desc* xd) { return (xd->w + 15) / 16; }
static int cin1_wtile_ne(const lamp_tensor_desc* xd) { return (18 * (16 * cin1_wtile_groups(xd) + 2) + 255) / 256; }
static bool cin1_wtile_ok(const lamp_tensor_desc* xd, const lamp_tensor_desc* dzd, const void* dz) {
    return (dzd->c == 32 || dzd->c == 64 || dzd->c == 128) && dzd->ldc % 8 == 0 && aligned16(dz) && cin1_wtile_ne(xd) <= 40 &&
           (int64_t)xd->n * xd->d * ((xd->h + 3) / 4) < ((int64_t)1 << 31);
}
static int cin1_wtile_gridx(const lamp_tensor_desc* xd) {
    const int64_t nblk = (int64_t)xd->n * xd->d * ((xd->h + 3) / 4);
    return (int)(nblk < 1024 ? nblk : 1024);
}
static size_t cin1_wtile_ws_bytes(const lamp_tensor_desc* xd, const lamp_tensor_desc* dzd) {
    return align_up((size_t)cin1_wtile_gridx(xd) * 4 * dzd->c * 27 * sizeof(float));
}
template <int CB>
static void cin1_wtile_launch(int ne, dim3 grid, size_t lds, hipStream_t s, const Cin1WArgs& a) {
    if (ne <= 12) hipLaunchKernelGGL((conv3d_cin1_wgrad_tile_kernel<CB, 12>), grid, dim3(256), lds, s, a);
    else if (ne <= 20) hipLaunchKernelGGL((conv3d_cin1_wgrad_tile_kernel<CB, 20>), grid, dim3(256), lds, s, a);
    else hipLaunchKernelGGL((conv3d_cin1_wgrad_tile_kernel<CB, 40>), grid, dim3(256), lds, s, a);
}
static lamp_status cin1_wtile(const lamp_tensor_desc* xd, const void* x, const lamp_tensor_desc* dzd, const void* dz, float* dw,
                              float beta, void* ws, size_t ws_bytes, hipStream_t s) {
    if (!ws || ws_bytes < cin1_wtile_ws_bytes(xd, dzd)) return LAMP_ERR_WORKSPACE;
    Cin1WArgs a;
    a.x = (const bf16_t*)x; a.ldx = xd->ldc; a.dz = (const bf16_t*)dz; a.lddz = dzd->ldc; a.part = (float*)ws;
    a.N = xd->n; a.D = xd->d; a.H = xd->h; a.W = xd->w; a.Co = dzd->c;
    a.G = cin1_wtile_groups(xd);
    a.WP = 16 * a.G + 2;
    a.RS = a.WP;
    {
        int l = 0;
        while ((1 << l) < a.WP) ++l;
        a.sWP = 31 + l;
        a.mWP = (uint32_t)((((uint64_t)1 << (31 + l)) + (uint64_t)a.WP - 1) / (uint64_t)a.WP);
    }
    const int cb = dzd->c >= 128 ? 4 : (dzd->c >= 64 ? 2 : 1);   // channels per workgroup column: 32 * cb
    const int gx = cin1_wtile_gridx(xd);
    const dim3 grid(gx, dzd->c / (32 * cb));
    const size_t lds = (size_t)4 * 2 * cb * 1024 + (size_t)18 * a.RS * sizeof(unsigned short);
    const int ne = cin1_wtile_ne(xd);
    if (cb == 1) cin1_wtile_launch<1>(ne, grid, lds, s, a);
    else if (cb == 2) cin1_wtile_launch<2>(ne, grid, lds, s, a);
    else cin1_wtile_launch<4>(ne, grid, lds, s, a);
    LAMP_CHECK_LAUNCH();
    return launch_reduce_partials((const float*)ws, gx * 4, (int64_t)dzd->c * 27, dw, beta, s);
}
static bool cin1_wgrad_ok(const lamp_tensor_desc* xd, const lamp_tensor_desc* dzd, const lamp_norm_in* xnorm) {
    const bool nm = xnorm && xnorm->mean_rstd && xnorm->c_norm > 0;
    return xd->dtype == LAMP_BF16 && xd->c == 1 && !nm && dzd->c % 32 == 0 && xd->w % 16 == 0 && nvox(xd) < ((int64_t)1 << 31);
}
// thread blocks (4 waves, one partial slab per wave) of the Cin == 1 weight gradient
static int cin1_wgrad_blocks(int64_t V) {
    int64_t b = (V / 16 + 3) / 4;
    return (int)(b > 2048 ? 2048 : (b < 1 ? 1 : b));
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

// The same sum with register tiling, for channel counts that are small multiples of 8 (the fp32 path of small
// nets): a thread owns OCG output channels of one voxel; the weights of a chunk of 8 input channels sit in
// LDS as [tap][ic][oc] (every lane of a wave reads the same few addresses), the input voxel is read once per
// (tap, ic) and used OCG times.  Input-channel chunks are taken in order, taps inside a chunk: a fixed order.
template <typename T, bool DGRAD, int OCG>
__global__ __launch_bounds__(256) void conv3d_regtile_kernel(const T* __restrict__ x, int ldx, const T* __restrict__ w,
                                                             const float* __restrict__ bias, T* __restrict__ z, int ldz, int N,
                                                             int D, int H, int W, int Cin, int Cout, int xvec, int wvec) {
    extern __shared__ float wsm[];   // [27][ICH][Cout]
    constexpr int ICH = 8;
    const int G = Cout / OCG, vpb = 256 / G;
    const int og = threadIdx.x % G, vl = threadIdx.x / G;
    const int64_t total = (int64_t)N * D * H * W;
    const int64_t v = (int64_t)blockIdx.x * vpb + vl;
    const bool active = vl < vpb && v < total;
    int wv = 0, h = 0, d = 0, n = 0;
    if (active) {
        wv = (int)(v % W);
        int64_t r = v / W;
        h = (int)(r % H);
        r /= H;
        d = (int)(r % D);
        n = (int)(r / D);
    }
    float acc[OCG];
#pragma unroll
    for (int o = 0; o < OCG; ++o) acc[o] = bias ? bias[og * OCG + o] : 0.f;
    for (int ic0 = 0; ic0 < Cin; ic0 += ICH) {
        const int nic = Cin - ic0 < ICH ? Cin - ic0 : ICH;
        __syncthreads();
        // weights of the chunk -> LDS [tap][ic][oc].  16-byte granules where the layout allows (forward: along ic,
        // the contiguous index of W[oc][t][ic]; data gradient: along oc of W[ic][26-t][oc]); four granules in flight.
        constexpr int VW = sizeof(T) == 2 ? 8 : 4;
        if (wvec && nic == ICH) {
            const int gtot = 27 * ICH * Cout / VW;
            for (int i0 = threadIdx.x; i0 < gtot; i0 += 1024) {
                float val[4][VW];
                int dst[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = i0 + 256 * u;
                    dst[u] = -1;
                    if (i < gtot) {
                        if (DGRAD) {
                            const int ocv = i % (Cout / VW), r = i / (Cout / VW), ic = r % ICH, t = r / ICH;
                            Vec<T, VW>::load(w + ((int64_t)(ic0 + ic) * 27 + (26 - t)) * Cout + ocv * VW, val[u]);
                            dst[u] = (t * ICH + ic) * Cout + ocv * VW;
                        } else {
                            const int icv = i % (ICH / VW), r = i / (ICH / VW), t = r % 27, oc = r / 27;
                            Vec<T, VW>::load(w + ((int64_t)oc * 27 + t) * Cin + ic0 + icv * VW, val[u]);
                            dst[u] = (t * ICH + icv * VW) * Cout + oc;
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (dst[u] >= 0) {
#pragma unroll
                        for (int e = 0; e < VW; ++e) wsm[dst[u] + (DGRAD ? e : e * Cout)] = val[u][e];
                    }
            }
        } else {
            const int wtot = 27 * nic * Cout;
            for (int i = threadIdx.x; i < wtot; i += 256) {
                const int ic = i % nic, r = i / nic;
                int t, oc;
                const T* src;
                if (DGRAD) {
                    oc = r % Cout; t = r / Cout;
                    src = w + ((int64_t)(ic0 + ic) * 27 + (26 - t)) * Cout + oc;
                } else {
                    t = r % 27; oc = r / 27;
                    src = w + ((int64_t)oc * 27 + t) * Cin + ic0 + ic;
                }
                wsm[(t * ICH + ic) * Cout + oc] = io<T>::ld(src);
            }
        }
        __syncthreads();
        if (!active) continue;
        // the three taps of a w-row are loaded together, one row ahead of the multiply-adds
        auto load_row = [&](int kdh, float (&xr)[3][ICH]) __attribute__((always_inline)) {
            const int id = d + kdh / 3 - 1, ih = h + kdh % 3 - 1;
            const bool rin = id >= 0 && id < D && ih >= 0 && ih < H;
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                const int iw = wv + kw - 1;
                const bool in = rin && iw >= 0 && iw < W;
                const T* xp = x + ((((int64_t)n * D + (rin ? id : d)) * H + (rin ? ih : h)) * W + (in ? iw : wv)) * ldx + ic0;
                if (xvec && nic == ICH) {   // one or two 16-byte loads instead of eight narrow ones
                    constexpr int VW = sizeof(T) == 2 ? 8 : 4;
                    if (in) {
                        Vec<T, VW>::load(xp, *reinterpret_cast<float(*)[VW]>(&xr[kw][0]));
                        if (VW == 4) Vec<T, VW>::load(xp + 4, *reinterpret_cast<float(*)[VW]>(&xr[kw][ICH - VW]));
                    } else {
#pragma unroll
                        for (int ic = 0; ic < ICH; ++ic) xr[kw][ic] = 0.f;
                    }
                } else {
#pragma unroll
                    for (int ic = 0; ic < ICH; ++ic) xr[kw][ic] = (in && ic < nic) ? io<T>::ld(xp + ic) : 0.f;
                }
            }
        };
        auto mul_row = [&](int kdh, const float (&xr)[3][ICH]) __attribute__((always_inline)) {
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                const float* wt = wsm + ((kdh * 3 + kw) * ICH) * Cout + og * OCG;
                if (nic == ICH) {   // branch-free: the eight weight rows are read ahead of the multiply-adds
                    float wr[ICH][OCG];
#pragma unroll
                    for (int ic = 0; ic < ICH; ++ic)
#pragma unroll
                        for (int o = 0; o < OCG; ++o) wr[ic][o] = wt[ic * Cout + o];
#pragma unroll
                    for (int ic = 0; ic < ICH; ++ic)
#pragma unroll
                        for (int o = 0; o < OCG; ++o) acc[o] = fmaf(xr[kw][ic], wr[ic][o], acc[o]);
                } else {
                    for (int ic = 0; ic < nic; ++ic)
#pragma unroll
                        for (int o = 0; o < OCG; ++o) acc[o] = fmaf(xr[kw][ic], wt[ic * Cout + o], acc[o]);
                }
            }
        };
        float xa[3][ICH], xb[3][ICH];
        load_row(0, xa);
#pragma unroll
        for (int kdh = 0; kdh < 9; kdh += 2) {
            if (kdh + 1 < 9) load_row(kdh + 1, xb);
            mul_row(kdh, xa);
            if (kdh + 2 < 9) load_row(kdh + 2, xa);
            if (kdh + 1 < 9) mul_row(kdh + 1, xb);
        }
    }
    if (active) {
#pragma unroll
        for (int o = 0; o < OCG; ++o) io<T>::st(z + v * ldz + og * OCG + o, acc[o]);
    }
}

template <bool DGRAD>
static lamp_status launch_direct(const lamp_tensor_desc* xd, const void* x, NormIn nm, const void* w, const float* bias,
                                 const lamp_tensor_desc* zd, void* z, hipStream_t s) {
    const int Cout = zd->c, Cin = xd->c;
    if (!nm.mean_rstd && Cout % 8 == 0 && Cout <= 64) {
        const int G = Cout / 8, vpb = 256 / G;
        const size_t shm = (size_t)27 * 8 * Cout * sizeof(float);   // at most 55 KB
        const dim3 grid(cdiv(nvox(zd), vpb));
        // 16-byte loads of a voxel's 8-channel chunk need aligned rows
        const int xvec = aligned16(x) && (xd->ldc * esize(xd->dtype)) % 16 == 0 ? 1 : 0;
        const int wvec = aligned16(w) && ((DGRAD ? Cout : Cin) * esize(xd->dtype)) % 16 == 0 ? 1 : 0;
        if (xd->dtype == LAMP_BF16)
            hipLaunchKernelGGL((conv3d_regtile_kernel<bf16_t, DGRAD, 8>), grid, dim3(256), shm, s, (const bf16_t*)x, xd->ldc,
                               (const bf16_t*)w, bias, (bf16_t*)z, zd->ldc, zd->n, zd->d, zd->h, zd->w, Cin, Cout, xvec, wvec);
        else
            hipLaunchKernelGGL((conv3d_regtile_kernel<float, DGRAD, 8>), grid, dim3(256), shm, s, (const float*)x, xd->ldc,
                               (const float*)w, bias, (float*)z, zd->ldc, zd->n, zd->d, zd->h, zd->w, Cin, Cout, xvec, wvec);
        LAMP_CHECK_LAUNCH();
        return LAMP_OK;
    }
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
    if (want_stats && xd->c == 1 && xd->dtype == LAMP_BF16 && cin1_tile_ok(zd)) {
        const size_t c = cin1_tile_ws_bytes(zd);
        if (c > a) a = c;
    }
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
        return mfma_conv_fwd(xd, x, w, false, zd, z, stats_out, eps, ws, ws_bytes, s, nullptr, bias, xnorm);
    if (cin1_fwd_ok(xd, zd, xnorm, bias, z)) {
        if (cin1_tile_ok(zd)) return cin1_tile_fwd(xd, x, w, zd, z, stats_out, eps, ws, ws_bytes, s);
        hipLaunchKernelGGL(conv3d_cin1_fwd_kernel, dim3(cdiv(nvox(zd), 256)), dim3(256), 0, s, (const bf16_t*)x, xd->ldc,
                           (const bf16_t*)w, (bf16_t*)z, zd->ldc, zd->n, zd->d, zd->h, zd->w, zd->c);
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

extern "C" size_t lamp_conv3d_dgrad_inorm_relu_bwd_workspace_bytes(const lamp_tensor_desc* dzd, const lamp_tensor_desc* gd) {
    if (!desc_ok(dzd) || !desc_ok(gd)) return 0;
    size_t b = lamp_conv3d_dgrad_workspace_bytes(dzd, gd);
    const size_t nb = lamp_inorm_relu_bwd_workspace_bytes(gd);
    if (nb > b) b = nb;
    if (mfma_conv_supported(dzd, gd, nullptr, nullptr)) {
        const size_t f = mfma_bsum_ws_bytes(dzd, gd) + align_up((size_t)gd->n * gd->c * 2 * sizeof(float));
        if (f > b) b = f;
    }
    return b;
}

extern "C" lamp_status lamp_conv3d_dgrad_inorm_relu_bwd(const lamp_tensor_desc* dzd, const void* dz, const void* w,
                                                        const lamp_tensor_desc* gd, void* g, const lamp_tensor_desc* zd,
                                                        const void* z, const float* stats, const float* gamma,
                                                        const float* beta, const lamp_tensor_desc* dzbd, void* dzb,
                                                        float* dgamma, float* dbeta, float beta_acc, void* ws,
                                                        size_t ws_bytes, void* stream) {
    lamp_status st = check_conv_pair(dzd, dz, gd, g);
    if (st != LAMP_OK) return st;
    if (!w || !zd || !z || !stats || !dzbd || !dzb) return LAMP_ERR_NULL;
    if (!desc_ok(zd) || !desc_ok(dzbd) || !same_space(gd, zd) || !same_space(gd, dzbd) || zd->c != gd->c || dzbd->c != gd->c)
        return LAMP_ERR_SHAPE;
    if (zd->dtype != gd->dtype || dzbd->dtype != gd->dtype) return LAMP_ERR_DTYPE;
    if (beta_acc != 0.f && beta_acc != 1.f) return LAMP_ERR_SHAPE;
    if (!ws || ws_bytes < lamp_conv3d_dgrad_inorm_relu_bwd_workspace_bytes(dzd, gd)) return LAMP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    if (mfma_bsum_supported(dzd, gd) && zd->ldc == gd->ldc && !(((uintptr_t)z) & 15u)) {
        // the sums at the tail of the workspace, the data gradient's own workspace in front of them
        const size_t cb = mfma_bsum_ws_bytes(dzd, gd);
        float* sums = (float*)((char*)ws + cb);
        ConvBsum bs{z, stats, gamma, beta, sums};
        st = mfma_conv_fwd(dzd, dz, w, true, gd, g, nullptr, 0.f, ws, cb, s, nullptr, nullptr, nullptr, &bs);
        if (st != LAMP_OK) return st;
        return launch_inorm_bwd_apply(gd, g, zd, z, stats, gamma, beta, sums, dzbd, dzb, dgamma, dbeta, beta_acc, s);
    }
    st = lamp_conv3d_dgrad(dzd, dz, w, gd, g, ws, ws_bytes, stream);
    if (st != LAMP_OK) return st;
    return lamp_inorm_relu_bwd(gd, g, zd, z, stats, gamma, beta, dzbd, dzb, dgamma, dbeta, beta_acc, ws, ws_bytes, stream);
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
    if (xd->dtype == LAMP_BF16 && xd->c == 1) {
        const size_t e = cin1_wtile_ws_bytes(xd, dzd);
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
    // The bias gradient's partial sums take the (256-byte aligned) head of the workspace, everything else what follows.
    const size_t cs = colsum_ws_bytes(nvox(dzd), dzd->c);
    if (dbias) {
        st = launch_colsum(dz, dzd->dtype, nvox(dzd), dzd->c, dzd->ldc, dbias, beta, ws, cs, s);
        if (st != LAMP_OK) return st;
    }
    ws = (char*)ws + cs;
    ws_bytes -= cs;
    if (mfma_wgrad_supported(xd, dzd, xnorm)) return mfma_wgrad(xd, x, dzd, dz, dw, beta, ws, ws_bytes, s);
    if (xd->dtype == LAMP_BF16 && xd->c == 1 && !(xnorm && xnorm->mean_rstd && xnorm->c_norm > 0) && cin1_wtile_ok(xd, dzd, dz))
        return cin1_wtile(xd, x, dzd, dz, dw, beta, ws, ws_bytes, s);
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
