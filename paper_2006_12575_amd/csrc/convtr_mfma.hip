// Matrix-core kernels for the 2x2x2 stride-2 transposed convolution (bf16, fp32 accumulate).
//
// Every output voxel depends on one input voxel and one tap, so forward and data gradient are plain
// GEMMs over voxels with a gather / scatter to the 2x2x2 sub-positions:
//   forward : Y[(tap,co)][v] = sum_ci  Wt'[(tap,co)][ci] * X[v][ci]        -> y[up(v,tap)][co]
//   dgrad   : DX[ci][v]      = sum_{(tap,co)} Wt[ci][(tap,co)] * DY[up(v,tap)][co]
// Operands are read straight from global memory into MFMA fragments (16 contiguous bytes per lane:
// the weights are small and cache-resident, the activations are streamed once); the op is bound by
// writing / reading the fine-resolution tensor, not by the matrix cores.
// The weight gradient has voxels as its reduction dimension and reads both operands through LDS with
// the transposing load, like the 3x3x3 weight gradient.
#include <stdlib.h>
#include "internal.h"

namespace lamp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;

struct CtArgs {
    const bf16_t* a;      // row-major A[rows][K]
    const bf16_t* b;      // activations (x for forward, dy for dgrad)
    bf16_t* out;
    const float* bias;    // forward only, [Co] or nullptr
    int rows, K;
    int N, D, H, W;       // coarse (input-resolution) dims
    int Ci, Co;
    int ldb, ldo;         // channel strides of b and out
    uint32_t mW, mH, mD;  // v / d == (v * m) >> s for v < 2^31 (round-up reciprocal, see ct_magic)
    int sW, sH, sD;
};

// wt'[(tap*Co + co)][ci] = wt[ci][tap][co]
__global__ __launch_bounds__(256) void convtr_repack_kernel(const bf16_t* __restrict__ wt, bf16_t* __restrict__ wp, int Ci,
                                                            int Co) {
    const int64_t total = (int64_t)Ci * 8 * Co;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int ci = (int)(i % Ci);
    const int r = (int)(i / Ci);  // tap*Co + co
    wp[i] = wt[(int64_t)ci * 8 * Co + r];
}

__device__ __forceinline__ bf16x8 gfrag(const bf16_t* p, bool ok) {
    uint4 q = make_uint4(0, 0, 0, 0);
    if (ok) q = *reinterpret_cast<const uint4*>(p);
    return __builtin_bit_cast(bf16x8, q);
}

// MODE 0: forward, MODE 1: data gradient.  One wave = 64 coarse voxels x up to 128 rows.
template <int MODE>
__global__ __launch_bounds__(256) void convtr_gemm_kernel(CtArgs a) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int64_t nvox = (int64_t)a.N * a.D * a.H * a.W;
    const int64_t v0 = ((int64_t)blockIdx.x * 4 + wv) * 64;
    if (v0 >= nvox) return;
    const int r0 = blockIdx.y * 128;
    const int nrb = min(4, (a.rows - r0 + 31) / 32);

    // the lane's two voxels (column j of voxel blocks 0 and 1) and their fine-resolution origin
    int64_t vq[2], fine[2];
    bool vok[2];
#pragma unroll
    for (int vb = 0; vb < 2; ++vb) {
        const int64_t v = v0 + vb * 32 + l32;
        vok[vb] = v < nvox;
        const int64_t vc = vok[vb] ? v : 0;
        const int w = (int)(vc % a.W);
        int64_t r = vc / a.W;
        const int h = (int)(r % a.H);
        r /= a.H;
        const int d = (int)(r % a.D);
        const int n = (int)(r / a.D);
        vq[vb] = vc;
        fine[vb] = (((int64_t)n * 2 * a.D + 2 * d) * 2 * a.H + 2 * h) * 2 * a.W + 2 * w;  // voxel (2d,2h,2w)
    }
    auto tap_off = [&](int tap) -> int64_t {
        const int i = tap >> 2, j = (tap >> 1) & 1, k = tap & 1;
        return ((int64_t)i * 2 * a.H + j) * 2 * a.W + k;
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int vb = 0; vb < 2; ++vb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rb][vb][r] = 0.f;

    for (int k0 = 0; k0 < a.K; k0 += 16) {
        const int k = k0 + 8 * half;
        bf16x8 bf[2], af[4];
        if (MODE == 0) {
#pragma unroll
            for (int vb = 0; vb < 2; ++vb) bf[vb] = gfrag(a.b + vq[vb] * a.ldb + k, vok[vb]);
        } else {
            const int tap = k / a.Co, co = k - tap * a.Co;
            const int64_t to = tap_off(tap);
#pragma unroll
            for (int vb = 0; vb < 2; ++vb) bf[vb] = gfrag(a.b + (fine[vb] + to) * a.ldb + co, vok[vb]);
        }
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) {
            const int row = r0 + rb * 32 + l32;
            af[rb] = gfrag(a.a + (int64_t)row * a.K + k, rb < nrb && row < a.rows);
        }
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
#pragma unroll
            for (int vb = 0; vb < 2; ++vb)
                if (rb < nrb) acc[rb][vb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[rb], bf[vb], acc[rb][vb], 0, 0, 0);
    }

    // lane holds, for its voxel of each block, rows r0 + rb*32 + 8*(r/4) + 4*half + (r%4)
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) {
        if (rb >= nrb) continue;
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            const int row = r0 + rb * 32 + rg * 8 + half * 4;
            if (row >= a.rows) continue;
#pragma unroll
            for (int vb = 0; vb < 2; ++vb) {
                if (!vok[vb]) continue;
                uint32_t pk[2];
                if (MODE == 0) {
                    const int tap = row / a.Co, co = row - tap * a.Co;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float bv = a.bias ? a.bias[co + e] : 0.f;
                        const uint32_t b = f2bf(acc[rb][vb][rg * 4 + e] + bv);
                        if (e & 1) pk[e >> 1] |= b << 16; else pk[e >> 1] = b;
                    }
                    *reinterpret_cast<uint2*>(a.out + (fine[vb] + tap_off(tap)) * a.ldo + co) = make_uint2(pk[0], pk[1]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint32_t b = f2bf(acc[rb][vb][rg * 4 + e]);
                        if (e & 1) pk[e >> 1] |= b << 16; else pk[e >> 1] = b;
                    }
                    *reinterpret_cast<uint2*>(a.out + vq[vb] * a.ldo + row) = make_uint2(pk[0], pk[1]);
                }
            }
        }
    }
}


// ------------------------------------------------------------------------------------------------
// Kernels for channel counts that are multiples of 32: the fine-resolution tensor is written
// (forward) and read (data gradient) in whole 64-byte pieces -- 32 channels of one fine voxel, four
// lanes of 16 bytes side by side -- instead of one 8-byte piece per lane.  A per-wave LDS buffer
// transposes between that memory order and the matrix-core fragment order; only the owning wave
// touches its buffer, so no workgroup barrier is needed.
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float ct_f32x2;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 ct_bf16x2;
__device__ __forceinline__ uint32_t ct_pack(float lo, float hi) {
    ct_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, ct_bf16x2));
}

static constexpr int CT_ROW = 80;  // bytes per voxel row in the transposing buffer: 64 of data, padded

// fine-resolution voxel (2d,2h,2w) of coarse voxel v (v < 2^31)
__device__ __forceinline__ uint32_t ct_div(uint32_t v, uint32_t m, int sh) { return (uint32_t)(((uint64_t)v * m) >> sh); }
__device__ __forceinline__ int64_t ct_fine_origin(const CtArgs& a, int64_t v) {
    const uint32_t vi = (uint32_t)v;
    uint32_t r = ct_div(vi, a.mW, a.sW);
    const uint32_t w = vi - r * (uint32_t)a.W;
    uint32_t r2 = ct_div(r, a.mH, a.sH);
    const uint32_t h = r - r2 * (uint32_t)a.H;
    const uint32_t n = ct_div(r2, a.mD, a.sD);
    const uint32_t d = r2 - n * (uint32_t)a.D;
    return (((int64_t)n * 2 * a.D + 2 * d) * 2 * a.H + 2 * h) * 2 * a.W + 2 * w;
}
__device__ __forceinline__ int64_t ct_tap_off(const CtArgs& a, int tap) {
    return ((int64_t)(tap >> 2) * 2 * a.H + ((tap >> 1) & 1)) * 2 * a.W + (tap & 1);
}

// Forward.  One wave = VB*32 coarse voxels x one block of RB units (a unit is (tap, 32 output
// channels) = 32 rows of the repacked weight).  With KS > 0 (K = 16*KS input channels) the wave's x
// operand is fetched up front in one go.  Every load of a wave is issued before its first store:
// loads and stores complete in one queue, so a load behind a store would wait for the store; the
// bias therefore sits in LDS.  Requires Co % 32 == 0, Co <= 256 * 4, Ci % 16 == 0, < 2^31 voxels.
template <int RB, int VB, int KS>
__global__ __launch_bounds__(256) void convtr_fwd32_kernel(CtArgs a) {
    constexpr int VW = 32 * VB;  // voxels per wave
    __shared__ __attribute__((aligned(16))) char tb[4][VW * CT_ROW];
    __shared__ __attribute__((aligned(16))) float bsh[4][1024];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int64_t nvox = (int64_t)a.N * a.D * a.H * a.W;
    const int K = KS > 0 ? 16 * KS : a.K;
    // workgroup id -> (voxel group, row block): ids are dealt round-robin to the 8 XCDs, so the row
    // blocks of one voxel group take consecutive slots of ONE XCD and share its L2 for x
    const int nblocks = a.rows / (32 * RB);
    const uint32_t xcd = blockIdx.x & 7u, slot = blockIdx.x >> 3;
    const int yb = (int)(slot % (uint32_t)nblocks);
    const int64_t vg = (int64_t)(slot / (uint32_t)nblocks) * 8 + xcd;
    const int64_t v0 = (vg * 4 + wv) * VW;
    if (v0 >= nvox) return;
    const int r0 = yb * (32 * RB);

    const bf16_t* xrow[VB];
#pragma unroll
    for (int vb = 0; vb < VB; ++vb) {
        int64_t v = v0 + vb * 32 + l32;  // columns past the end repeat the last voxel and are never stored
        if (v >= nvox) v = nvox - 1;
        xrow[vb] = a.b + v * a.ldb + 8 * half;
    }
    const bf16_t* arow = a.a + (int64_t)(r0 + l32) * K + 8 * half;
    bf16x8 ball[KS > 0 ? KS : 1][VB];
    if (KS > 0) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int vb = 0; vb < VB; ++vb) ball[ks][vb] = *reinterpret_cast<const bf16x8*>(xrow[vb] + ks * 16);
    }
    // bias -> this wave's LDS copy
    for (int c = lane * 4; c < a.Co; c += 256) {
        float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
        if (a.bias) bv = make_float4(a.bias[c], a.bias[c + 1], a.bias[c + 2], a.bias[c + 3]);
        *reinterpret_cast<float4*>(&bsh[wv][c]) = bv;
    }
    // the voxels this lane stores: 16 per pass, four lanes per voxel
    int64_t fs[2 * VB];
#pragma unroll
    for (int it = 0; it < 2 * VB; ++it) {
        const int64_t v = v0 + it * 16 + (lane >> 2);
        fs[it] = v < nvox ? ct_fine_origin(a, v) : -1;
    }

    f32x16 acc[RB][VB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int vb = 0; vb < VB; ++vb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rb][vb][r] = 0.f;

    if (KS > 0) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bf16x8 af[RB];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) af[rb] = *reinterpret_cast<const bf16x8*>(arow + rb * 32 * K + ks * 16);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int vb = 0; vb < VB; ++vb)
                    acc[rb][vb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[rb], ball[ks][vb], acc[rb][vb], 0, 0, 0);
        }
    } else {
        // streaming reduction, operands fetched one step ahead
        bf16x8 bfn[VB], afn[RB];
#pragma unroll
        for (int vb = 0; vb < VB; ++vb) bfn[vb] = *reinterpret_cast<const bf16x8*>(xrow[vb]);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) afn[rb] = *reinterpret_cast<const bf16x8*>(arow + (int64_t)rb * 32 * K);
        for (int k0 = 0; k0 < K; k0 += 16) {
            bf16x8 bf[VB], af[RB];
#pragma unroll
            for (int vb = 0; vb < VB; ++vb) bf[vb] = bfn[vb];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) af[rb] = afn[rb];
            if (k0 + 16 < K) {
#pragma unroll
                for (int vb = 0; vb < VB; ++vb) bfn[vb] = *reinterpret_cast<const bf16x8*>(xrow[vb] + k0 + 16);
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) afn[rb] = *reinterpret_cast<const bf16x8*>(arow + (int64_t)rb * 32 * K + k0 + 16);
            }
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int vb = 0; vb < VB; ++vb)
                    acc[rb][vb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[rb], bf[vb], acc[rb][vb], 0, 0, 0);
        }
    }

    // lane holds, for voxel l32 of block vb, rows 8*(r/4) + 4*half + (r%4) of the unit
    char* mine = tb[wv];
    const int cpt = a.Co >> 5;
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int unit = (r0 >> 5) + rb;
        const int tap = unit / cpt, co0 = (unit - tap * cpt) << 5;
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            const int c = rg * 8 + half * 4;
            const float4 bv = *reinterpret_cast<const float4*>(&bsh[wv][co0 + c]);
#pragma unroll
            for (int vb = 0; vb < VB; ++vb) {
                const uint2 pk = make_uint2(ct_pack(acc[rb][vb][rg * 4 + 0] + bv.x, acc[rb][vb][rg * 4 + 1] + bv.y),
                                            ct_pack(acc[rb][vb][rg * 4 + 2] + bv.z, acc[rb][vb][rg * 4 + 3] + bv.w));
                *reinterpret_cast<uint2*>(mine + (vb * 32 + l32) * CT_ROW + c * 2) = pk;
            }
        }
        __builtin_amdgcn_wave_barrier();
        const int64_t to = ct_tap_off(a, tap);
#pragma unroll
        for (int it = 0; it < 2 * VB; ++it) {
            const uint4 q = *reinterpret_cast<const uint4*>(mine + (it * 16 + (lane >> 2)) * CT_ROW + (lane & 3) * 16);
            if (fs[it] >= 0) *reinterpret_cast<uint4*>(a.out + (fs[it] + to) * a.ldo + co0 + (lane & 3) * 8) = q;
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// Data gradient.  One wave = 64 coarse voxels x RB blocks of 32 input channels; the reduction runs
// over units of (tap, 32 output channels).  The 64-byte pieces of dy are gathered one unit ahead
// into registers and handed to the matrix-core fragment order through the wave's double buffer.
// Requires Co % 32 == 0, Ci % 32 == 0.
template <int RB>
__global__ __launch_bounds__(256) void convtr_dgrad32_kernel(CtArgs a) {
    __shared__ __attribute__((aligned(16))) char tb[4][2][64 * CT_ROW];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int64_t nvox = (int64_t)a.N * a.D * a.H * a.W;
    const int64_t v0 = ((int64_t)blockIdx.x * 4 + wv) * 64;
    if (v0 >= nvox) return;
    const int r0 = blockIdx.y * (32 * RB);
    const int nrb = min(RB, (a.rows - r0) >> 5);

    int64_t fs[4], vs[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        vs[it] = v0 + it * 16 + (lane >> 2);
        fs[it] = vs[it] < nvox ? ct_fine_origin(a, vs[it]) : -1;
    }
    const bf16_t* arow = a.a + (int64_t)(r0 + l32) * a.K + 8 * half;
    const int cpt = a.Co >> 5, units = 8 * cpt;

    auto gather = [&](int u, uint4 (&q)[4]) {
        const int tap = u / cpt, c0 = (u - tap * cpt) << 5;
        const int64_t to = ct_tap_off(a, tap);
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            q[it] = make_uint4(0, 0, 0, 0);
            if (fs[it] >= 0) q[it] = *reinterpret_cast<const uint4*>(a.b + (fs[it] + to) * a.ldb + c0 + (lane & 3) * 8);
        }
    };
    auto put = [&](char* buf, const uint4 (&q)[4]) {
#pragma unroll
        for (int it = 0; it < 4; ++it) *reinterpret_cast<uint4*>(buf + (it * 16 + (lane >> 2)) * CT_ROW + (lane & 3) * 16) = q[it];
    };

    f32x16 acc[RB][2];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int vb = 0; vb < 2; ++vb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rb][vb][r] = 0.f;

    uint4 q[4];
    gather(0, q);
    put(tb[wv][0], q);
    __builtin_amdgcn_wave_barrier();
    for (int u = 0; u < units; ++u) {
        if (u + 1 < units) gather(u + 1, q);
        const char* cur = tb[wv][u & 1];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 bf[2], af[RB];
#pragma unroll
            for (int vb = 0; vb < 2; ++vb)
                bf[vb] = *reinterpret_cast<const bf16x8*>(cur + (vb * 32 + l32) * CT_ROW + ks * 32 + half * 16);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) af[rb] = gfrag(arow + (int64_t)rb * 32 * a.K + u * 32 + ks * 16, rb < nrb);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int vb = 0; vb < 2; ++vb)
                    if (rb < nrb) acc[rb][vb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[rb], bf[vb], acc[rb][vb], 0, 0, 0);
        }
        if (u + 1 < units) put(tb[wv][(u + 1) & 1], q);
        __builtin_amdgcn_wave_barrier();
    }

    char* mine = tb[wv][0];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        if (rb >= nrb) break;
#pragma unroll
        for (int rg = 0; rg < 4; ++rg)
#pragma unroll
            for (int vb = 0; vb < 2; ++vb) {
                const uint2 pk = make_uint2(ct_pack(acc[rb][vb][rg * 4 + 0], acc[rb][vb][rg * 4 + 1]),
                                            ct_pack(acc[rb][vb][rg * 4 + 2], acc[rb][vb][rg * 4 + 3]));
                *reinterpret_cast<uint2*>(mine + (vb * 32 + l32) * CT_ROW + (rg * 8 + half * 4) * 2) = pk;
            }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const uint4 o = *reinterpret_cast<const uint4*>(mine + (it * 16 + (lane >> 2)) * CT_ROW + (lane & 3) * 16);
            if (vs[it] < nvox) *reinterpret_cast<uint4*>(a.out + vs[it] * a.ldo + r0 + rb * 32 + (lane & 3) * 8) = o;
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// round-up reciprocal for exact division of v < 2^31 by d: v / d == (v * m) >> s
static void ct_magic(int d, uint32_t* m, int* s) {
    int l = 0;
    while ((1ll << l) < d) ++l;
    *s = 31 + l;
    *m = (uint32_t)((((uint64_t)1 << (31 + l)) + (uint64_t)d - 1) / (uint64_t)d);
}
static void ct_set_magic(CtArgs& a) {
    ct_magic(a.W, &a.mW, &a.sW);
    ct_magic(a.H, &a.mH, &a.sH);
    ct_magic(a.D, &a.mD, &a.sD);
}

// 32 rows per wave when the volume is small (more workgroups), up to 128 otherwise (measured: from 32768
// voxels on the fewer re-reads of dy win)
static int ct_row_blocks(int64_t nv, int rows) {
    if (nv < 32768) return 1;
    return rows >= 128 ? 4 : (rows >= 64 ? 2 : 1);
}

bool mfma_convtr_supported(const lamp_tensor_desc* xd, const lamp_tensor_desc* yd, const lamp_norm_in* xnorm) {
    if (xd->dtype != LAMP_BF16) return false;
    if (xnorm && xnorm->mean_rstd && xnorm->c_norm > 0) return false;
    if (xd->c % 16 || yd->c % 8 || xd->ldc % 8 || yd->ldc % 4) return false;
    return true;
}

size_t mfma_convtr_ws_bytes(const lamp_tensor_desc* xd, const lamp_tensor_desc* yd) {
    if (!mfma_convtr_supported(xd, yd, nullptr)) return 0;
    return align_up((size_t)xd->c * 8 * yd->c * 2);
}

lamp_status mfma_convtr_fwd(const lamp_tensor_desc* xd, const void* x, const void* wt, const float* bias,
                            const lamp_tensor_desc* yd, void* y, void* ws, size_t ws_bytes, hipStream_t s) {
    if ((((uintptr_t)x) & 15u) || (((uintptr_t)y) & 7u) || (((uintptr_t)ws) & 15u)) return LAMP_ERR_ALIGN;
    if (ws_bytes < mfma_convtr_ws_bytes(xd, yd)) return LAMP_ERR_WORKSPACE;
    const int Ci = xd->c, Co = yd->c;
    bf16_t* wp = (bf16_t*)ws;
    hipLaunchKernelGGL(convtr_repack_kernel, dim3(cdiv((int64_t)Ci * 8 * Co, 256)), dim3(256), 0, s, (const bf16_t*)wt, wp, Ci, Co);
    LAMP_CHECK_LAUNCH();
    CtArgs a;
    a.a = wp; a.b = (const bf16_t*)x; a.out = (bf16_t*)y; a.bias = bias; a.rows = 8 * Co; a.K = Ci;
    a.N = xd->n; a.D = xd->d; a.H = xd->h; a.W = xd->w; a.Ci = Ci; a.Co = Co; a.ldb = xd->ldc; a.ldo = yd->ldc;
    if (Co % 32 == 0 && Co <= 1024 && yd->ldc % 8 == 0 && ((((uintptr_t)y) & 15u) == 0) && nvox(xd) < ((int64_t)1 << 31)) {
        const int64_t nv = nvox(xd);
        ct_set_magic(a);
        if (Ci >= 256) {
            // many input channels: a wave takes 64 voxels x 8 units (16 accumulator tiles), so that every weight
            // fragment fetched from the cache feeds two matrix-core instructions and the row blocks re-read x less
            dim3 grid((unsigned)(cdiv(cdiv(nv, 256), 8) * 8 * (a.rows / 256)));
            hipLaunchKernelGGL((convtr_fwd32_kernel<8, 2, 0>), grid, dim3(256), 0, s, a);
        } else if (nv >= 65536) {
            // a wave = 32 voxels x 8 units: for Co = 32 it writes all eight taps of its voxels
            const int64_t groups8 = cdiv(cdiv(nv, 128), 8) * 8;  // voxel groups, padded to whole XCD rounds
            dim3 grid((unsigned)(groups8 * (a.rows / 256)));
            if (Ci == 64) hipLaunchKernelGGL((convtr_fwd32_kernel<8, 1, 4>), grid, dim3(256), 0, s, a);
            else if (Ci == 128) hipLaunchKernelGGL((convtr_fwd32_kernel<8, 1, 8>), grid, dim3(256), 0, s, a);
            else hipLaunchKernelGGL((convtr_fwd32_kernel<8, 1, 0>), grid, dim3(256), 0, s, a);
        } else {
            const int64_t groups8 = cdiv(cdiv(nv, 256), 8) * 8;
            dim3 grid((unsigned)(groups8 * (a.rows / 32)));
            hipLaunchKernelGGL((convtr_fwd32_kernel<1, 2, 0>), grid, dim3(256), 0, s, a);
        }
        LAMP_CHECK_LAUNCH();
        return LAMP_OK;
    }
    dim3 grid(cdiv(nvox(xd), 256), cdiv(a.rows, 128));
    hipLaunchKernelGGL((convtr_gemm_kernel<0>), grid, dim3(256), 0, s, a);
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}

bool mfma_convtr_dgrad_supported(const lamp_tensor_desc* xd, const lamp_tensor_desc* dyd, const lamp_tensor_desc* dxd) {
    if (xd->dtype != LAMP_BF16) return false;
    if (xd->c % 4 || dyd->c % 8 || dyd->ldc % 8 || dxd->ldc % 4) return false;
    return true;
}

lamp_status mfma_convtr_dgrad(const lamp_tensor_desc* xd, const void* wt, const lamp_tensor_desc* dyd, const void* dy,
                              const lamp_tensor_desc* dxd, void* dx, hipStream_t s) {
    if ((((uintptr_t)dy) & 15u) || (((uintptr_t)dx) & 7u) || (((uintptr_t)wt) & 15u)) return LAMP_ERR_ALIGN;
    CtArgs a;
    a.a = (const bf16_t*)wt; a.b = (const bf16_t*)dy; a.out = (bf16_t*)dx; a.bias = nullptr; a.rows = xd->c; a.K = 8 * dyd->c;
    a.N = xd->n; a.D = xd->d; a.H = xd->h; a.W = xd->w; a.Ci = xd->c; a.Co = dyd->c; a.ldb = dyd->ldc; a.ldo = dxd->ldc;
    if (a.Co % 32 == 0 && a.Ci % 32 == 0 && dyd->ldc % 8 == 0 && dxd->ldc % 8 == 0 && ((((uintptr_t)dx) & 15u) == 0) &&
        nvox(xd) < ((int64_t)1 << 31)) {
        ct_set_magic(a);
        const int rb = ct_row_blocks(nvox(xd), a.rows);
        dim3 grid(cdiv(nvox(xd), 256), cdiv(a.rows, 32 * rb));
        if (rb == 4) hipLaunchKernelGGL((convtr_dgrad32_kernel<4>), grid, dim3(256), 0, s, a);
        else if (rb == 2) hipLaunchKernelGGL((convtr_dgrad32_kernel<2>), grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL((convtr_dgrad32_kernel<1>), grid, dim3(256), 0, s, a);
        LAMP_CHECK_LAUNCH();
        return LAMP_OK;
    }
    dim3 grid(cdiv(nvox(xd), 256), cdiv(a.rows, 128));
    hipLaunchKernelGGL((convtr_gemm_kernel<1>), grid, dim3(256), 0, s, a);
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}

// ------------------------------------------------------------------------------------------------
// Weight gradient  dWt[ci][tap][co] = sum_v x[v][ci] * dy[up(v,tap)][co]   (K = coarse voxels).
// Workgroup = 4 waves on (split s, 64-wide ci block, 32-wide co block); wave w owns taps 2w, 2w+1.
// Chunks of 64 coarse voxels are staged in LDS (x rows of 128 bytes, dy rows of 64 bytes per tap,
// double buffered, register-free copies) and read with the transposing LDS load.
// (inline assembly, so that the compiler's wait-count bookkeeping does not see the copies and keeps
// partial waits for the fragment reads; completion is tracked by hand)
__device__ __forceinline__ void g2lds16_ct(const void* g, char* lds_base) {
    const uint32_t m = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds_base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(m), "v"(g) : "memory", "m0");
}
template <int ROWB> __device__ __forceinline__ bf16x8 frag_tr(const char* p) {
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * ROWB));
    typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

struct CtWArgs {
    const bf16_t* x; int ldx;
    const bf16_t* dy; int ldy;
    float* part;              // [S][Ci][8][Co]
    const bf16_t* zero16;
    int N, D, H, W, Ci, Co;
    int chunks_per_split;     // 64-voxel chunks per split
};

static constexpr int CTW_X = 64 * 128;            // x tile bytes
static constexpr int CTW_DY = 8 * 64 * 64;        // dy tile bytes (8 taps)
static constexpr int CTW_STAGE = CTW_X + CTW_DY;  // 40960

__device__ __forceinline__ void ctw_stage(const CtWArgs& a, char* __restrict__ st, int64_t v0, int64_t nvox, int ci0,
                                          int co0, int wv, int lane) {
    // x: copy q = wv*2 + i covers voxels 8q..8q+7, 8 pieces of 16 bytes each
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int q = wv * 2 + i;
        const int64_t v = v0 + q * 8 + (lane >> 3);
        const int pc = lane & 7;
        const bool ok = v < nvox && ci0 + pc * 8 < a.Ci;
        g2lds16_ct(ok ? a.x + v * a.ldx + ci0 + pc * 8 : a.zero16, st + q * 1024);
    }
    // dy: copy q = wv*8 + i: tap q/4, voxels 16*(q%4) .. +15, 4 pieces each
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int q = wv * 8 + i;
        const int tap = q >> 2;
        const int64_t v = v0 + (q & 3) * 16 + (lane >> 2);
        const int pc = lane & 3;
        const bf16_t* src = a.zero16;
        if (v < nvox) {
            const int vi = (int)v;  // host guarantees nvox < 2^31
            const int w = vi % a.W;
            int r = vi / a.W;
            const int h = r % a.H;
            r /= a.H;
            const int d = r % a.D, n = r / a.D;
            const int64_t ov = (((int64_t)n * 2 * a.D + 2 * d + (tap >> 2)) * 2 * a.H + 2 * h + ((tap >> 1) & 1)) * 2 * a.W + 2 * w + (tap & 1);
            src = a.dy + ov * a.ldy + co0 + pc * 8;
        }
        g2lds16_ct(src, st + CTW_X + q * 1024);
    }
}

__device__ __forceinline__ void ctw_compute(f32x16 (&acc)[2][2], const char* __restrict__ st, int wv, int lane) {
    const int b16 = lane >> 4, s16 = lane & 15;
    const uint32_t lx = (uint32_t)((8 * (b16 >> 1) + (s16 >> 2)) * 128 + 32 * (b16 & 1) + 8 * (s16 & 3));
    const uint32_t ly = (uint32_t)((8 * (b16 >> 1) + (s16 >> 2)) * 64 + 32 * (b16 & 1) + 8 * (s16 & 3));
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        bf16x8 af[2], bf[2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) af[rb] = frag_tr<128>(st + ks * 16 * 128 + rb * 64 + lx);
#pragma unroll
        for (int t = 0; t < 2; ++t) bf[t] = frag_tr<64>(st + CTW_X + ((wv * 2 + t) * 64 + ks * 16) * 64 + ly);
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int t = 0; t < 2; ++t) acc[rb][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[rb], bf[t], acc[rb][t], 0, 0, 0);
    }
}

__global__ __launch_bounds__(256) void convtr_wgrad_mfma_kernel(CtWArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int ci0 = blockIdx.y * 64, co0 = blockIdx.z * 32;
    const int64_t nvox = (int64_t)a.N * a.D * a.H * a.W;
    const int64_t nchunks = (nvox + 63) / 64;
    const int64_t c_lo = (int64_t)blockIdx.x * a.chunks_per_split;
    int64_t c_hi = c_lo + a.chunks_per_split;
    if (c_hi > nchunks) c_hi = nchunks;
    f32x16 acc[2][2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rb][t][r] = 0.f;
    if (c_lo < c_hi) ctw_stage(a, lds, c_lo * 64, nvox, ci0, co0, wv, lane);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    int par = 0;
    for (int64_t c = c_lo; c < c_hi; ++c, par ^= 1) {
        if (c + 1 < c_hi) ctw_stage(a, lds + (par ^ 1) * CTW_STAGE, (c + 1) * 64, nvox, ci0, co0, wv, lane);
        __builtin_amdgcn_sched_barrier(0);
        ctw_compute(acc, lds + par * CTW_STAGE, wv, lane);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    }
    float* pb = a.part + (int64_t)blockIdx.x * a.Ci * 8 * a.Co;
    const int l32 = lane & 31, half = lane >> 5;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ci = ci0 + rb * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                if (ci < a.Ci) pb[((int64_t)ci * 8 + wv * 2 + t) * a.Co + co0 + l32] = acc[rb][t][r];
            }
}


static int ctw_splits(const lamp_tensor_desc* xd, const lamp_tensor_desc* dyd) {
    const int64_t chunks = (nvox(xd) + 63) / 64;
    const int types = ((xd->c + 63) / 64) * (dyd->c / 32);
    int64_t s = 512 / types;  // about two workgroups per CU; more only enlarges the partial sums
    if (s < 1) s = 1;
    if (s > chunks) s = chunks;
    return (int)s;
}

bool mfma_convtr_wgrad_supported(const lamp_tensor_desc* xd, const lamp_tensor_desc* dyd, const lamp_norm_in* xnorm) {
    if (xd->dtype != LAMP_BF16) return false;
    if (xnorm && xnorm->mean_rstd && xnorm->c_norm > 0) return false;
    if (xd->c % 32 || dyd->c % 32 || xd->ldc % 8 || dyd->ldc % 8) return false;
    if (nvox(xd) >= ((int64_t)1 << 31)) return false;
    return true;
}

size_t mfma_convtr_wgrad_ws_bytes(const lamp_tensor_desc* xd, const lamp_tensor_desc* dyd) {
    if (!mfma_convtr_wgrad_supported(xd, dyd, nullptr)) return 0;
    return align_up((size_t)ctw_splits(xd, dyd) * xd->c * 8 * dyd->c * sizeof(float)) + 256;
}

lamp_status mfma_convtr_wgrad(const lamp_tensor_desc* xd, const void* x, const lamp_tensor_desc* dyd, const void* dy,
                              float* dwt, float beta, void* ws, size_t ws_bytes, hipStream_t s) {
    if ((((uintptr_t)x) & 15u) || (((uintptr_t)dy) & 15u) || (((uintptr_t)ws) & 15u)) return LAMP_ERR_ALIGN;
    if (ws_bytes < mfma_convtr_wgrad_ws_bytes(xd, dyd)) return LAMP_ERR_WORKSPACE;
    const int S = ctw_splits(xd, dyd);
    const int64_t O = (int64_t)xd->c * 8 * dyd->c;
    CtWArgs a;
    a.x = (const bf16_t*)x; a.ldx = xd->ldc; a.dy = (const bf16_t*)dy; a.ldy = dyd->ldc; a.part = (float*)ws;
    const bool direct = S == 1 && beta == 0.f;   // the only partial is the result: written in place
    if (direct) a.part = dwt;
    a.zero16 = device_zero16();
    if (!a.zero16) return LAMP_ERR_HIP;
    a.N = xd->n; a.D = xd->d; a.H = xd->h; a.W = xd->w; a.Ci = xd->c; a.Co = dyd->c;
    const int64_t chunks = (nvox(xd) + 63) / 64;
    a.chunks_per_split = (int)((chunks + S - 1) / S);
    if (ensure_dyn_lds((const void*)convtr_wgrad_mfma_kernel, 2 * CTW_STAGE) != LAMP_OK) return LAMP_ERR_HIP;
    dim3 grid(S, (xd->c + 63) / 64, dyd->c / 32);
    hipLaunchKernelGGL(convtr_wgrad_mfma_kernel, grid, dim3(256), 2 * CTW_STAGE, s, a);
    LAMP_CHECK_LAUNCH();
    if (direct) return LAMP_OK;
    return launch_reduce_partials((const float*)ws, S, O, dwt, beta, s);
}

}  // namespace lamp
