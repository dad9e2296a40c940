// Matrix-core (MFMA) implicit-GEMM 3x3x3 convolution kernels for gfx950, bf16 in / fp32 accumulate.
//
// Forward and data-gradient share one kernel (the data gradient is a forward convolution with
// spatially flipped taps and swapped channel roles, done by the weight repack).
//
// GEMM view per workgroup tile:  D[co][voxel] += sum_{tap, ci} Wp[tap][co][ci] * X[voxel + tap][ci]
//   M = 32*COB output channels (A operand = weights), N = 512 voxels (B operand = activations),
//   K = 27 taps x Cin, walked as (Cin chunk of 32) x (9 tap groups of 3) x (2 k-steps of 16).
// Tile: 4 x 8 x 16 output voxels (d,h,w); wave w of the 4 owns d-slice w = 4 blocks of 32 voxels
// (2 h-rows x 16 w), so a 16-lane group always reads 16 consecutive halo voxels from LDS.
// LDS: two halo buffers (6 x 10 x 18 voxels x 32 channels, 64-byte rows, XOR-swizzled 16-byte parts)
// so the next chunk / next tile streams in while the current one is multiplied, and two small
// weight buffers (3 taps x 64 co x 32 ci).  Workgroups are persistent and walk an XCD-contiguous
// range of tiles.
#include "internal.h"

namespace lamp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

static constexpr int TD = 4, TH = 8, TW = 16;
static constexpr int HD = TD + 2, HH = TH + 2, HW = TW + 2;
static constexpr int HALO_VOX = HD * HH * HW;          // 1080
static constexpr int HALO_BYTES = HALO_VOX * 64;       // one 32-channel chunk
static constexpr int HALO_PIECES = HALO_VOX * 4;       // 16-byte pieces
static constexpr int HALO_ITERS = (HALO_PIECES + 255) / 256;  // 17
static constexpr int PIECES_PER_GROUP = 2;             // 9 groups x 2 >= 17
static constexpr int WBUF_BYTES = 3 * 64 * 64;         // 3 taps x 64 co x 32 ci bf16
static constexpr int LDS_BYTES = 2 * HALO_BYTES + 2 * WBUF_BYTES;

__device__ __forceinline__ uint32_t swz(uint32_t row) { return (row >> 2) & 3u; }

__device__ __forceinline__ bf16x8 lds_frag(const char* p) {
    uint4 q = *reinterpret_cast<const uint4*>(p);
    return __builtin_bit_cast(bf16x8, q);
}

// wp[t][oc][ic]  <-  forward: W[oc][t][ic]     dgrad: W[ic][26-t][oc]
__global__ __launch_bounds__(256) void repack_weights_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wp,
                                                             int Cout, int Cin, int dgrad) {
    const int64_t total = (int64_t)27 * Cout * Cin;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int ic = (int)(i % Cin);
    const int oc = (int)((i / Cin) % Cout);
    const int t = (int)(i / ((int64_t)Cin * Cout));
    wp[i] = dgrad ? w[((int64_t)ic * 27 + (26 - t)) * Cout + oc] : w[((int64_t)oc * 27 + t) * Cin + ic];
}

struct ConvArgs {
    const bf16_t* x; int ldx;
    const bf16_t* wp;
    bf16_t* z; int ldz;
    float* part;        // [N][tiles_per_n][Cout][2] or nullptr
    int N, D, H, W, Cin, Cout;
    int tiles_d, tiles_h, tiles_w, tiles_per_n, tiles_total, tiles_per_xcd;
};

template <int COB>
__global__ __launch_bounds__(256) void conv3d_igemm_kernel(ConvArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char* hbuf0 = lds;
    char* wbuf0 = lds + 2 * HALO_BYTES;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int co0 = blockIdx.y * (32 * COB);
    const int nchunks = a.Cin >> 5;

    // persistent walk over an XCD-contiguous range of tiles
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3, wg_per_xcd = gridDim.x >> 3;
    const int tile_lo = xcd * a.tiles_per_xcd;
    const int tile_hi = min(tile_lo + a.tiles_per_xcd, a.tiles_total);

    // ---- per-lane constants of the fragment reads
    // A (weights): row = co within the 64-row buffer; part = ks*2 + half
    uint32_t a_off[2];
    {
        const uint32_t s = swz((uint32_t)l32);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) a_off[ks] = (uint32_t)l32 * 64u + ((((uint32_t)(ks * 2 + half)) ^ s) << 4);
    }
    // B (activations): halo row of this lane's voxel in block vb, tap (0,0,0)
    const int bw = l32 & 15, bh = l32 >> 4;
    const uint32_t hv_base = (uint32_t)((wv * HH + bh) * HW + bw);

    // ---- staging helpers
    auto halo_piece_load = [&](int p, int tile, int chunk, uint4& v) {
        v = make_uint4(0, 0, 0, 0);
        if (p < HALO_PIECES) {
            const int hv = p >> 2, part = p & 3;
            const int hw = hv % HW, hh = (hv / HW) % HH, hd = hv / (HW * HH);
            const int n = tile / a.tiles_per_n;
            int r = tile - n * a.tiles_per_n;
            const int tw = r % a.tiles_w;
            r /= a.tiles_w;
            const int th = r % a.tiles_h, tdd = r / a.tiles_h;
            const int gd = tdd * TD + hd - 1, gh = th * TH + hh - 1, gw = tw * TW + hw - 1;
            if (gd >= 0 && gd < a.D && gh >= 0 && gh < a.H && gw >= 0 && gw < a.W) {
                const bf16_t* src = a.x + ((((int64_t)n * a.D + gd) * a.H + gh) * a.W + gw) * a.ldx + chunk * 32 + part * 8;
                v = *reinterpret_cast<const uint4*>(src);
            }
        }
    };
    auto halo_piece_store = [&](int p, char* hb, const uint4& v) {
        if (p < HALO_PIECES) {
            const uint32_t hv = (uint32_t)p >> 2, part = (uint32_t)p & 3u;
            *reinterpret_cast<uint4*>(hb + hv * 64u + ((part ^ swz(hv)) << 4)) = v;
        }
    };
    // weights of tap group g (taps 3g..3g+2) of a chunk: 3 x (32*COB) rows x 4 parts
    constexpr int WPIECES = 3 * 32 * COB * 4;
    constexpr int WITERS = (WPIECES + 255) / 256;
    auto w_piece_load = [&](int i, int g, int chunk, uint4& v) {
        const int p = tid + i * 256;
        if (p < WPIECES) {
            const int part = p & 3, row = (p >> 2) % (32 * COB), t = p / (4 * 32 * COB);
            const bf16_t* src = a.wp + ((int64_t)(3 * g + t) * a.Cout + co0 + row) * a.Cin + chunk * 32 + part * 8;
            v = *reinterpret_cast<const uint4*>(src);
        }
    };
    auto w_piece_store = [&](int i, char* wb, const uint4& v) {
        const int p = tid + i * 256;
        if (p < WPIECES) {
            const uint32_t part = p & 3, row = (p >> 2) % (32 * COB), t = p / (4 * 32 * COB);
            *reinterpret_cast<uint4*>(wb + (t * 64u + row) * 64u + ((part ^ swz(row)) << 4)) = v;
        }
    };

    int tile = tile_lo + local;
    if (tile >= tile_hi) return;

    // ---- prologue: first halo chunk and first weight group, synchronously
    for (int i = 0; i < HALO_ITERS; ++i) {
        uint4 v;
        halo_piece_load(tid + i * 256, tile, 0, v);
        halo_piece_store(tid + i * 256, hbuf0, v);
    }
    for (int i = 0; i < WITERS; ++i) {
        uint4 v;
        w_piece_load(i, 0, 0, v);
        w_piece_store(i, wbuf0, v);
    }
    __syncthreads();

    int stage = 0;  // parity selects the halo buffer
    int wpar = 0;   // parity selects the weight buffer
    for (; tile < tile_hi; tile += wg_per_xcd) {
        f32x16 acc[COB][4];
#pragma unroll
        for (int cb = 0; cb < COB; ++cb)
#pragma unroll
            for (int vb = 0; vb < 4; ++vb)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[cb][vb][r] = 0.f;

        const int next_tile = tile + wg_per_xcd;
        for (int chunk = 0; chunk < nchunks; ++chunk, ++stage) {
            const char* hb = hbuf0 + (stage & 1) * HALO_BYTES;
            char* hb_next = hbuf0 + ((stage + 1) & 1) * HALO_BYTES;
            // what streams in during this stage
            const bool last_chunk = chunk + 1 == nchunks;
            const int pf_tile = last_chunk ? next_tile : tile;
            const int pf_chunk = last_chunk ? 0 : chunk + 1;
            const bool pf = !last_chunk || next_tile < tile_hi;
#pragma unroll 1
            for (int g = 0; g < 9; ++g, wpar ^= 1) {
                const char* wb = wbuf0 + wpar * WBUF_BYTES;
                char* wb_next = wbuf0 + (wpar ^ 1) * WBUF_BYTES;
                // issue the global loads of this group's share of the prefetch
                uint4 hp[PIECES_PER_GROUP], wpv[WITERS];
                if (pf) {
#pragma unroll
                    for (int i = 0; i < PIECES_PER_GROUP; ++i)
                        halo_piece_load(tid + (g * PIECES_PER_GROUP + i) * 256, pf_tile, pf_chunk, hp[i]);
                }
                // next weight group: (chunk, g+1), or (next stage, 0)
                const bool wlast = g == 8;
                const bool wpf = !wlast || pf;
                if (wpf) {
#pragma unroll
                    for (int i = 0; i < WITERS; ++i) w_piece_load(i, wlast ? 0 : g + 1, wlast ? pf_chunk : chunk, wpv[i]);
                }
                // ---- multiply: 3 taps x 2 k-steps
                const int kd = g / 3, kh = g - 3 * kd;
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) {
                    const uint32_t tapoff = (uint32_t)(kd * HH * HW + kh * HW + kw);
                    bf16x8 af[COB][2], bfr[4][2];
#pragma unroll
                    for (int cb = 0; cb < COB; ++cb)
#pragma unroll
                        for (int ks = 0; ks < 2; ++ks) af[cb][ks] = lds_frag(wb + (kw * 64 + cb * 32) * 64 + a_off[ks]);
#pragma unroll
                    for (int vb = 0; vb < 4; ++vb) {
                        const uint32_t hv = hv_base + (uint32_t)(vb * 2 * HW) + tapoff;
                        const uint32_t s = swz(hv);
#pragma unroll
                        for (int ks = 0; ks < 2; ++ks)
                            bfr[vb][ks] = lds_frag(hb + hv * 64u + ((((uint32_t)(ks * 2 + half)) ^ s) << 4));
                    }
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                        for (int cb = 0; cb < COB; ++cb)
#pragma unroll
                            for (int vb = 0; vb < 4; ++vb)
                                acc[cb][vb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[cb][ks], bfr[vb][ks], acc[cb][vb], 0, 0, 0);
                }
                // ---- land the prefetched pieces
                if (pf) {
#pragma unroll
                    for (int i = 0; i < PIECES_PER_GROUP; ++i)
                        halo_piece_store(tid + (g * PIECES_PER_GROUP + i) * 256, hb_next, hp[i]);
                }
                if (wpf) {
#pragma unroll
                    for (int i = 0; i < WITERS; ++i) w_piece_store(i, wb_next, wpv[i]);
                }
                __syncthreads();
            }
        }

        // ---- epilogue: bf16 store of z and per-tile channel sums of the stored values
        const int n = tile / a.tiles_per_n;
        int r0 = tile - n * a.tiles_per_n;
        const int tw = r0 % a.tiles_w;
        r0 /= a.tiles_w;
        const int th = r0 % a.tiles_h, tdd = r0 / a.tiles_h;
        const int gd = tdd * TD + wv;
        float ssum[COB][16], ssq[COB][16];
#pragma unroll
        for (int cb = 0; cb < COB; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) { ssum[cb][r] = 0.f; ssq[cb][r] = 0.f; }
#pragma unroll
        for (int vb = 0; vb < 4; ++vb) {
            const int gh = th * TH + vb * 2 + bh, gw = tw * TW + bw;
            const bool ok = gd < a.D && gh < a.H && gw < a.W;
            bf16_t* zp = a.z + ((((int64_t)n * a.D + gd) * a.H + gh) * a.W + gw) * a.ldz + co0 + 4 * half;
#pragma unroll
            for (int cb = 0; cb < COB; ++cb)
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    uint32_t pk[2];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const bf16_t b = f2bf(acc[cb][vb][rg * 4 + e]);
                        const float fv = ok ? bf2f(b) : 0.f;
                        ssum[cb][rg * 4 + e] += fv;
                        ssq[cb][rg * 4 + e] = fmaf(fv, fv, ssq[cb][rg * 4 + e]);
                        if (e & 1) pk[e >> 1] |= ((uint32_t)b) << 16; else pk[e >> 1] = b;
                    }
                    if (ok) *reinterpret_cast<uint2*>(zp + cb * 32 + rg * 8) = make_uint2(pk[0], pk[1]);
                }
        }
        if (a.part) {
            // reduce over the 32 lanes that share `half` (xor 1,2,4,8,16), then across the 4 waves
            // scratch: the halo buffer of the stage just finished (free until the next stage's prefetch)
            float* sred = reinterpret_cast<float*>(hbuf0 + ((stage + 1) & 1) * HALO_BYTES);
#pragma unroll
            for (int cb = 0; cb < COB; ++cb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float s = ssum[cb][r], q = ssq[cb][r];
#pragma unroll
                    for (int m = 1; m < 32; m <<= 1) {
                        s += __shfl_xor(s, m);
                        q += __shfl_xor(q, m);
                    }
                    if (l32 == 0) {
                        const int c = cb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
                        sred[(wv * 64 + c) * 2 + 0] = s;
                        sred[(wv * 64 + c) * 2 + 1] = q;
                    }
                }
            __syncthreads();
            if (tid < 32 * COB * 2) {
                const int c = tid >> 1, k = tid & 1;
                const float v = sred[(0 * 64 + c) * 2 + k] + sred[(1 * 64 + c) * 2 + k] + sred[(2 * 64 + c) * 2 + k] +
                                sred[(3 * 64 + c) * 2 + k];
                a.part[(((int64_t)n * a.tiles_per_n + (tile - n * a.tiles_per_n)) * a.Cout + co0 + c) * 2 + k] = v;
            }
            __syncthreads();
        }
    }
}

// counts[p] = voxels of tile p that lie inside the volume (same for every sample)
__global__ void tile_counts_kernel(int32_t* counts, int D, int H, int W, int tiles_d, int tiles_h, int tiles_w) {
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= tiles_d * tiles_h * tiles_w) return;
    const int tw = p % tiles_w, th = (p / tiles_w) % tiles_h, tdd = p / (tiles_w * tiles_h);
    const int d = min(TD, D - tdd * TD), h = min(TH, H - th * TH), w = min(TW, W - tw * TW);
    counts[p] = d * h * w;
}

static void tile_dims(const lamp_tensor_desc* t, int& td, int& th, int& tw) {
    td = (t->d + TD - 1) / TD; th = (t->h + TH - 1) / TH; tw = (t->w + TW - 1) / TW;
}

bool mfma_conv_supported(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd, const lamp_norm_in* xnorm,
                         const float* bias) {
    if (xd->dtype != LAMP_BF16) return false;
    if (xnorm && xnorm->mean_rstd && xnorm->c_norm > 0) return false;
    if (bias) return false;
    if (xd->c % 32 || zd->c % 32 || xd->ldc % 8 || zd->ldc % 4) return false;
    return true;
}

size_t mfma_conv_ws_bytes(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd, int want_stats) {
    if (!mfma_conv_supported(xd, zd, nullptr, nullptr)) return 0;
    int td, th, tw;
    tile_dims(zd, td, th, tw);
    const size_t tiles = (size_t)td * th * tw;
    size_t b = align_up((size_t)27 * xd->c * zd->c * 2);
    if (want_stats) b += align_up((size_t)zd->n * tiles * zd->c * 2 * sizeof(float)) + align_up(tiles * sizeof(int32_t));
    return b;
}

lamp_status mfma_conv_fwd(const lamp_tensor_desc* xd, const void* x, const void* w, bool dgrad,
                          const lamp_tensor_desc* zd, void* z, float* stats_out, float eps, void* ws, size_t ws_bytes,
                          hipStream_t s) {
    if ((((uintptr_t)x) & 15u) || (((uintptr_t)z) & 7u) || (((uintptr_t)ws) & 15u)) return LAMP_ERR_ALIGN;
    int td, th, tw;
    tile_dims(zd, td, th, tw);
    const int tiles_per_n = td * th * tw;
    Carver cv(ws, ws_bytes);
    bf16_t* wp = (bf16_t*)cv.take((size_t)27 * xd->c * zd->c * 2);
    float* part = nullptr;
    int32_t* counts = nullptr;
    if (stats_out) {
        part = (float*)cv.take((size_t)zd->n * tiles_per_n * zd->c * 2 * sizeof(float));
        counts = (int32_t*)cv.take((size_t)tiles_per_n * sizeof(int32_t));
    }
    if (!cv.ok()) return LAMP_ERR_WORKSPACE;
    const int64_t wtotal = (int64_t)27 * xd->c * zd->c;
    hipLaunchKernelGGL(repack_weights_kernel, dim3(cdiv(wtotal, 256)), dim3(256), 0, s, (const bf16_t*)w, wp, zd->c, xd->c,
                       dgrad ? 1 : 0);
    LAMP_CHECK_LAUNCH();
    ConvArgs a;
    a.x = (const bf16_t*)x; a.ldx = xd->ldc; a.wp = wp; a.z = (bf16_t*)z; a.ldz = zd->ldc; a.part = part;
    a.N = zd->n; a.D = zd->d; a.H = zd->h; a.W = zd->w; a.Cin = xd->c; a.Cout = zd->c;
    a.tiles_d = td; a.tiles_h = th; a.tiles_w = tw; a.tiles_per_n = tiles_per_n;
    a.tiles_total = tiles_per_n * zd->n;
    a.tiles_per_xcd = (a.tiles_total + 7) / 8;
    const int cob = (zd->c % 64 == 0) ? 2 : 1;
    int wgx = 256;  // one persistent workgroup per CU (LDS-limited), 32 per XCD
    while (wgx > 8 && (wgx / 8) > a.tiles_per_xcd) wgx -= 8;
    const size_t shm = LDS_BYTES;
    dim3 grid(wgx, zd->c / (32 * cob));
    static bool attr_done[2] = {false, false};
    if (cob == 2) {
        if (!attr_done[1]) {
            if (hipFuncSetAttribute((const void*)conv3d_igemm_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm) != hipSuccess)
                return LAMP_ERR_HIP;
            attr_done[1] = true;
        }
        hipLaunchKernelGGL((conv3d_igemm_kernel<2>), grid, dim3(256), shm, s, a);
    } else {
        if (!attr_done[0]) {
            if (hipFuncSetAttribute((const void*)conv3d_igemm_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm) != hipSuccess)
                return LAMP_ERR_HIP;
            attr_done[0] = true;
        }
        hipLaunchKernelGGL((conv3d_igemm_kernel<1>), grid, dim3(256), shm, s, a);
    }
    LAMP_CHECK_LAUNCH();
    if (stats_out) {
        hipLaunchKernelGGL(tile_counts_kernel, dim3(cdiv(tiles_per_n, 256)), dim3(256), 0, s, counts, zd->d, zd->h, zd->w, td,
                           th, tw);
        LAMP_CHECK_LAUNCH();
        return launch_stats_finalize(part, counts, tiles_per_n, zd->n, zd->c, eps, stats_out, s);
    }
    return LAMP_OK;
}

// ------------------------------------------------------------------------------------------------
// Weight gradient:  dW[co][tap][ci] = sum_v dz[v][co] * x[v + tap][ci]
//
// GEMM view: M = co (A = dz^T), N = ci (B = x shifted by the tap), K = voxels.  Both operands are
// needed K-major per lane but live channel-major (NDHWC) in LDS, so fragments are read with the
// transposing LDS load (ds_read_b64_tr_b16): inside each 16-lane group, source lane s supplies
// 4 channels of voxel row s/4 and lane t receives channel t of 4 consecutive voxel rows.
// A workgroup (8 waves) owns one 32-wide ci block and 32*COB output channels for all 27 taps, the
// taps dealt round-robin to the waves (<= 4 each, accumulators 2*4*16 registers), and walks a
// contiguous range of 2 x 8 x 16 voxel tiles, accumulating in registers; tiles are double
// buffered in LDS.  Per-workgroup partials are summed by a second, fixed-order kernel.
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;

static constexpr int WTD = 2, WTH = 8, WTW = 16;
static constexpr int WHD = WTD + 2, WHH = WTH + 2, WHW = WTW + 2;
static constexpr int WTILE_VOX = WTD * WTH * WTW;             // 256
static constexpr int WX_VOX = WHD * WHH * WHW;                // 720
static constexpr int WX_BYTES = WX_VOX * 64;                  // 32 ci per row
static constexpr int WDZ_HALF_BYTES = WTILE_VOX * 64;         // one 32-co half, 64-byte rows
static constexpr int WBUF_STAGE = WX_BYTES + 2 * WDZ_HALF_BYTES;  // 78848
static constexpr int WG_LDS_BYTES = 2 * WBUF_STAGE;           // 157696

struct WgradArgs {
    const bf16_t* x; int ldx;
    const bf16_t* dz; int lddz;
    float* part;  // [S][Cout][27][Cin]
    int N, D, H, W, Cin, Cout;
    int tiles_d, tiles_h, tiles_w, tiles_per_n, tiles_total, tiles_per_wg;
};

__device__ __forceinline__ bf16x8 lds_frag_tr(const char* p) {
    // two transposing loads: voxel rows +0..3 and +4..7 (4 rows of 64 bytes further on)
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 256));
    typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

template <int COB>
__global__ __launch_bounds__(512) void conv3d_wgrad_kernel(WgradArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int ci0 = blockIdx.y * 32, co0 = blockIdx.z * (32 * COB);
    const int tile_lo = blockIdx.x * a.tiles_per_wg;
    const int tile_hi = min(tile_lo + a.tiles_per_wg, a.tiles_total);

    // taps of this wave: wv, wv+8, wv+16, wv+24 (the last only for waves 0..2)
    uint32_t tapoff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = wv + 8 * i;
        const int kd = t / 9, kh = (t / 3) % 3, kw = t % 3;
        tapoff[i] = (uint32_t)(((kd * WHH + kh) * WHW + kw) * 64);
    }
    const bool has4 = wv + 24 < 27;

    // lane part of a transposing fragment read: voxel row 8*(b/2) + s/4, channel bytes 32*(b%2) + 8*(s%4)
    const int b16 = lane >> 4, s16 = lane & 15;
    const uint32_t loff = (uint32_t)((8 * (b16 >> 1) + (s16 >> 2)) * 64 + 32 * (b16 & 1) + 8 * (s16 & 3));

    f32x16 acc[COB][4];
#pragma unroll
    for (int cb = 0; cb < COB; ++cb)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[cb][i][r] = 0.f;

    // ---- staging: 16-byte pieces.  dz: 256 voxels x (4*COB) pieces ; x: 720 voxels x 4 pieces
    constexpr int DZ_PIECES = WTILE_VOX * 4 * COB;
    constexpr int DZ_ITERS = DZ_PIECES / 512;          // 4 (COB=2) or 2
    constexpr int X_PIECES = WX_VOX * 4;               // 2880
    constexpr int X_ITERS = (X_PIECES + 511) / 512;    // 6
    auto tile_coords = [&](int tile, int& n, int& d0, int& h0, int& w0) {
        n = tile / a.tiles_per_n;
        int r = tile - n * a.tiles_per_n;
        w0 = (r % a.tiles_w) * WTW;
        r /= a.tiles_w;
        h0 = (r % a.tiles_h) * WTH;
        d0 = (r / a.tiles_h) * WTD;
    };
    auto dz_load = [&](int i, int tile, uint4& v) {
        const int p = tid + i * 512;
        const int part = p % (4 * COB), vx = p / (4 * COB);
        const int w = vx % WTW, h = (vx / WTW) % WTH, d = vx / (WTW * WTH);
        int n, d0, h0, w0;
        tile_coords(tile, n, d0, h0, w0);
        const int gd = d0 + d, gh = h0 + h, gw = w0 + w;
        v = make_uint4(0, 0, 0, 0);
        if (gd < a.D && gh < a.H && gw < a.W)
            v = *reinterpret_cast<const uint4*>(a.dz + ((((int64_t)n * a.D + gd) * a.H + gh) * a.W + gw) * a.lddz + co0 + part * 8);
    };
    auto dz_store = [&](int i, char* st, const uint4& v) {
        const int p = tid + i * 512;
        const int part = p % (4 * COB), vx = p / (4 * COB);
        // 32-co half (part / 4) in its own array of 64-byte rows
        *reinterpret_cast<uint4*>(st + WX_BYTES + (part >> 2) * WDZ_HALF_BYTES + vx * 64 + (part & 3) * 16) = v;
    };
    auto x_load = [&](int i, int tile, uint4& v) {
        const int p = tid + i * 512;
        v = make_uint4(0, 0, 0, 0);
        if (p < X_PIECES) {
            const int part = p & 3, hv = p >> 2;
            const int hw = hv % WHW, hh = (hv / WHW) % WHH, hd = hv / (WHW * WHH);
            int n, d0, h0, w0;
            tile_coords(tile, n, d0, h0, w0);
            const int gd = d0 + hd - 1, gh = h0 + hh - 1, gw = w0 + hw - 1;
            if (gd >= 0 && gd < a.D && gh >= 0 && gh < a.H && gw >= 0 && gw < a.W)
                v = *reinterpret_cast<const uint4*>(a.x + ((((int64_t)n * a.D + gd) * a.H + gh) * a.W + gw) * a.ldx + ci0 + part * 8);
        }
    };
    auto x_store = [&](int i, char* st, const uint4& v) {
        const int p = tid + i * 512;
        if (p < X_PIECES) *reinterpret_cast<uint4*>(st + (p >> 2) * 64 + (p & 3) * 16) = v;
    };

    if (tile_lo < tile_hi) {
        // prologue: first tile synchronously
        for (int i = 0; i < DZ_ITERS; ++i) { uint4 v; dz_load(i, tile_lo, v); dz_store(i, lds, v); }
        for (int i = 0; i < X_ITERS; ++i) { uint4 v; x_load(i, tile_lo, v); x_store(i, lds, v); }
    }
    __syncthreads();

    int par = 0;
    for (int tile = tile_lo; tile < tile_hi; ++tile, par ^= 1) {
        const char* st = lds + par * WBUF_STAGE;
        char* st_next = lds + (par ^ 1) * WBUF_STAGE;
        const bool pf = tile + 1 < tile_hi;
        const char* xb = st + loff;
        const char* dzb = st + WX_BYTES + loff;
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
            // first half of the k-steps carries the dz prefetch, second half the x prefetch
            uint4 pv[X_ITERS];
            if (pf) {
                if (hf == 0) {
#pragma unroll
                    for (int i = 0; i < DZ_ITERS; ++i) dz_load(i, tile + 1, pv[i]);
                } else {
#pragma unroll
                    for (int i = 0; i < X_ITERS; ++i) x_load(i, tile + 1, pv[i]);
                }
            }
#pragma unroll
            for (int k8 = 0; k8 < 8; ++k8) {
                const int ks = hf * 8 + k8;            // k-step = one 16-voxel w-row: d = ks/8, h = ks%8
                const int d = ks >> 3, h = ks & 7;
                bf16x8 af[COB], bfr[4];
#pragma unroll
                for (int cb = 0; cb < COB; ++cb) af[cb] = lds_frag_tr(dzb + cb * WDZ_HALF_BYTES + ks * 16 * 64);
                const uint32_t rowoff = (uint32_t)((d * WHH + h) * WHW * 64);
#pragma unroll
                for (int i = 0; i < 3; ++i) bfr[i] = lds_frag_tr(xb + rowoff + tapoff[i]);
                if (has4) bfr[3] = lds_frag_tr(xb + rowoff + tapoff[3]);
#pragma unroll
                for (int i = 0; i < 3; ++i)
#pragma unroll
                    for (int cb = 0; cb < COB; ++cb)
                        acc[cb][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[cb], bfr[i], acc[cb][i], 0, 0, 0);
                if (has4) {
#pragma unroll
                    for (int cb = 0; cb < COB; ++cb)
                        acc[cb][3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[cb], bfr[3], acc[cb][3], 0, 0, 0);
                }
            }
            if (pf) {
                if (hf == 0) {
#pragma unroll
                    for (int i = 0; i < DZ_ITERS; ++i) dz_store(i, st_next, pv[i]);
                } else {
#pragma unroll
                    for (int i = 0; i < X_ITERS; ++i) x_store(i, st_next, pv[i]);
                }
            }
        }
        __syncthreads();
    }

    // ---- write this workgroup's partial: part[slot][co][tap][ci]
    float* pb = a.part + (int64_t)blockIdx.x * a.Cout * 27 * a.Cin;
    const int l32 = lane & 31, half = lane >> 5;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = wv + 8 * i;
        if (t < 27) {
#pragma unroll
            for (int cb = 0; cb < COB; ++cb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int co = co0 + cb * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                    pb[((int64_t)co * 27 + t) * a.Cin + ci0 + l32] = acc[cb][i][r];
                }
        }
    }
}

static void wtile_dims(const lamp_tensor_desc* t, int& td, int& th, int& tw) {
    td = (t->d + WTD - 1) / WTD; th = (t->h + WTH - 1) / WTH; tw = (t->w + WTW - 1) / WTW;
}

static int wgrad_slots(const lamp_tensor_desc* xd, const lamp_tensor_desc* dzd) {
    int td, th, tw;
    wtile_dims(xd, td, th, tw);
    const int64_t tiles = (int64_t)td * th * tw * xd->n;
    const int cob = (dzd->c % 64 == 0) ? 2 : 1;
    const int types = (xd->c / 32) * (dzd->c / (32 * cob));
    int64_t s = 256 / types;
    if (s < 1) s = 1;
    if (s >= 8) s = s / 8 * 8;  // keep the types of one tile range on one XCD
    if (s > tiles) s = tiles;
    return (int)s;
}

bool mfma_wgrad_supported(const lamp_tensor_desc* xd, const lamp_tensor_desc* dzd, const lamp_norm_in* xnorm) {
    if (xd->dtype != LAMP_BF16) return false;
    if (xnorm && xnorm->mean_rstd && xnorm->c_norm > 0) return false;
    if (xd->c % 32 || dzd->c % 32 || xd->ldc % 8 || dzd->ldc % 8) return false;
    return true;
}

size_t mfma_wgrad_ws_bytes(const lamp_tensor_desc* xd, const lamp_tensor_desc* dzd) {
    if (!mfma_wgrad_supported(xd, dzd, nullptr)) return 0;
    return align_up((size_t)wgrad_slots(xd, dzd) * dzd->c * 27 * xd->c * sizeof(float));
}

lamp_status mfma_wgrad(const lamp_tensor_desc* xd, const void* x, const lamp_tensor_desc* dzd, const void* dz, float* dw,
                       float beta, void* ws, size_t ws_bytes, hipStream_t s) {
    if ((((uintptr_t)x) & 15u) || (((uintptr_t)dz) & 15u) || (((uintptr_t)ws) & 15u)) return LAMP_ERR_ALIGN;
    if (ws_bytes < mfma_wgrad_ws_bytes(xd, dzd)) return LAMP_ERR_WORKSPACE;
    WgradArgs a;
    a.x = (const bf16_t*)x; a.ldx = xd->ldc; a.dz = (const bf16_t*)dz; a.lddz = dzd->ldc; a.part = (float*)ws;
    a.N = xd->n; a.D = xd->d; a.H = xd->h; a.W = xd->w; a.Cin = xd->c; a.Cout = dzd->c;
    wtile_dims(xd, a.tiles_d, a.tiles_h, a.tiles_w);
    a.tiles_per_n = a.tiles_d * a.tiles_h * a.tiles_w;
    a.tiles_total = a.tiles_per_n * xd->n;
    const int S = wgrad_slots(xd, dzd);
    a.tiles_per_wg = (a.tiles_total + S - 1) / S;
    const int cob = (dzd->c % 64 == 0) ? 2 : 1;
    dim3 grid(S, xd->c / 32, dzd->c / (32 * cob));
    static bool attr_done[2] = {false, false};
    if (cob == 2) {
        if (!attr_done[1]) {
            if (hipFuncSetAttribute((const void*)conv3d_wgrad_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, WG_LDS_BYTES) != hipSuccess)
                return LAMP_ERR_HIP;
            attr_done[1] = true;
        }
        hipLaunchKernelGGL((conv3d_wgrad_kernel<2>), grid, dim3(512), WG_LDS_BYTES, s, a);
    } else {
        if (!attr_done[0]) {
            if (hipFuncSetAttribute((const void*)conv3d_wgrad_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, WG_LDS_BYTES) != hipSuccess)
                return LAMP_ERR_HIP;
            attr_done[0] = true;
        }
        hipLaunchKernelGGL((conv3d_wgrad_kernel<1>), grid, dim3(512), WG_LDS_BYTES, s, a);
    }
    LAMP_CHECK_LAUNCH();
    return launch_reduce_partials((const float*)ws, S, (int64_t)dzd->c * 27 * xd->c, dw, beta, s);
}

}  // namespace lamp
