// Matrix-core implicit-GEMM 3x3x3 convolution, "ring" variant: bf16 in / fp32 accumulate, gfx950.
//
// Same GEMM view as the tiled kernel (D[co][voxel] += Wp[tap][co][ci] * X[voxel + tap][ci]; forward and
// data gradient differ only in the weight repack), but organised so that every input byte is fetched
// from memory once per tile and every LDS fragment feeds as many MFMAs as possible:
//
//  * Tile = 4 x 8 x 16 output voxels, 4 waves (one per SIMD).  A wave owns 4 d-slices x (2 h-rows x 16 w)
//    = four 32-voxel blocks for all 32*COB output channels.  For a fixed in-plane tap (kh,kw) the input
//    slice s = d + kd serves output slices d = s, s-1, s-2 with the weights of kd = 0, 1, 2: six slice
//    fragments and 3*COB weight fragments feed 12*COB MFMAs.
//  * LDS holds a ring of 3 halo regions, each one 16-channel chunk of a tile's 6 x 10 x 18 halo (two
//    planes of 16-byte voxel entries), and a ring of 9 weight blocks (3 taps x 16 ci x 32*COB co).
//    Region (q+2)%3 is refilled for chunk-step q+2 while chunk-step q is multiplied, weight block s%9
//    for step s+9 while step s is multiplied, both by register-free global -> LDS copies.  Copies
//    complete in issue order, so the long weight ring is what lets a halo copy that misses every
//    cache stay in flight for 7 steps without holding up the weights behind it.
//  * One step = one (chunk, kh, kw); a barrier per step publishes the copies two steps ahead of their
//    use, so fragment reads for step s+1 are issued inside step s and the MFMA stream never drains.
//  * A persistent workgroup walks a run of tiles that is contiguous in d, so the two halo slices shared
//    by successive tiles are re-read from cache soon after their first use.
#include <stdlib.h>
#include "internal.h"

namespace lamp {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int RTD = 4, RTH = 8, RTW = 16;
constexpr int RHD = RTD + 2, RHH = RTH + 2, RHW = RTW + 2;
constexpr int RHALO_VOX = RHD * RHH * RHW;   // 1080
constexpr int RPLANE = RHALO_VOX * 16;       // 8 channels per voxel entry
constexpr int RREGION = 2 * RPLANE;          // one 16-channel chunk: 34560
constexpr int RNREG = 3;
constexpr int RSLICE = RHH * RHW * 16;       // bytes between halo d-slices of a plane
constexpr int RHENTRIES = 2 * RHALO_VOX;     // 16-byte entries of a region: 36 wave copies, 9 per wave, copy k
constexpr int RHSTEP = 60;                   // starts at entry min(60k, 2160-64) (neighbours overlap by 4 entries)
constexpr int RNWSLOT = 9;                  // weight ring: block of step s + 9 replaces block s
constexpr int RINFLIGHT = 7;                // steps whose copies may still be in flight at a step's end
constexpr int REPI_STORES = 16;             // output stores a wave issues in the epilogue of a tile inside the volume

template <int COB> struct RW {
    static constexpr int WROWS = 32 * COB;
    static constexpr int WPLANE = WROWS * 16;        // one (tap, plane): WROWS rows of 16 bytes
    static constexpr int WBLOCK = 6 * WPLANE;        // 3 taps (kd) x 2 planes
    static constexpr int WBLOCK_ELEMS = WBLOCK / 2;
    static constexpr int WENTRIES = 6 * WROWS;       // 16-byte entries of a block: 8 wave copies, 2 per wave, copy u
    static constexpr int USTEP = WENTRIES / 8;       // starts at entry min(u * USTEP, WENTRIES - 64)
    static constexpr int LDS_BYTES = RNREG * RREGION + RNWSLOT * WBLOCK;
};

struct RingArgs {
    const bf16_t* x; int ldx;
    const bf16_t* wp;
    bf16_t* z; int ldz;
    float* part;           // [N][tiles_per_n][Cout][2] or nullptr
    int32_t* counts;       // [tiles_per_n] in-volume voxels per tile (written when part != nullptr)
    const bf16_t* zero16;  // 16 zero bytes in global memory (source of the zero padding)
    int N, D, H, W, Cin, Cout;
    int tiles_d, tiles_h, tiles_w, tiles_per_n, tiles_total, tiles_per_xcd, tiles_per_wg;
};

__device__ __forceinline__ bf16x8 lds_frag(const char* p) {
    uint4 q = *reinterpret_cast<const uint4*>(p);
    return __builtin_bit_cast(bf16x8, q);
}
// 16-byte global -> LDS copy that bypasses registers: lane l's 16 bytes land at lds_base + 16*l
// (lds_base must be wave-uniform); inactive lanes write nothing.  Issued as inline assembly so that
// the compiler's wait-count bookkeeping does not see it: with the builtin form every later wait for an
// LDS fragment read degrades to "wait for all reads", which stalls the MFMA stream.  Completion is
// tracked by hand with wait_vmcnt.
__device__ __forceinline__ void g2lds16(const void* g, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(g) : "memory", "m0");
}
// Two floats to a pair of bf16 (round to nearest even) with the hardware conversion.
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
template <int K, int NM, int NR> __device__ __forceinline__ void sched_interleave() {
    if constexpr (K < NM) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        constexpr int R = (NR * (K + 1)) / NM - (NR * K) / NM;
        if constexpr (R > 0) __builtin_amdgcn_sched_group_barrier(0x100, R, 0);
        sched_interleave<K + 1, NM, NR>();
    }
}
template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// wp[slab][chunk][kh*3+kw][kd][plane][co in slab][8]  <-  forward: W[oc][t][ic]   dgrad: W[ic][26-t][oc]
// (t = kd*9 + kh*3 + kw, ic = chunk*16 + plane*8 + e): the weight block of every step is contiguous and
// the steps of a tile follow each other in memory.
__global__ __launch_bounds__(256) void ring_repack_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wp, int Cout,
                                                          int Cin, int wrows, int dgrad) {
    const int64_t total = (int64_t)27 * Cout * Cin;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < 8) wp[total + i] = 0;  // 16 zero bytes behind the weights: the source of the zero padding
    if (i >= total) return;
    const int nchunks = Cin >> 4;
    int64_t r = i;
    const int e = (int)(r % 8); r /= 8;
    const int co = (int)(r % wrows); r /= wrows;
    const int plane = (int)(r % 2); r /= 2;
    const int kd = (int)(r % 3); r /= 3;
    const int j = (int)(r % 9); r /= 9;
    const int chunk = (int)(r % nchunks);
    const int slab = (int)(r / nchunks);
    const int oc = slab * wrows + co, ic = chunk * 16 + plane * 8 + e, t = kd * 9 + j;
    wp[i] = dgrad ? w[((int64_t)ic * 27 + (26 - t)) * Cout + oc] : w[((int64_t)oc * 27 + t) * Cin + ic];
}

struct HaloTile {
    const bf16_t* origin;              // x at the halo origin (d0-1, h0-1, w0-1) of the tile (may be out of range)
    int dlo, dhi, hlo, hhi, wlo, whi;  // halo coords inside the volume: lo <= c <= hi
};

// ---- one step = in-plane tap J = kh*3 + kw of the current chunk: 12*COB MFMAs, 6 + 3*COB fragment
// reads (3 slices of this step, then the weights and the first 3 slices of the next step) and 3 copies.
// With one wave per SIMD nothing else hides a stall, so the instruction order is fixed by hand: the
// step is cut into slots of one MFMA each, every read, copy and piece of address arithmetic is
// assigned to a slot, and a scheduling fence closes each slot.
template <int COB> struct StepPlan {
    static constexpr int NM = 12 * COB, NR = 6 + 3 * COB;
    struct M { int s, kd, cb; };
    // MFMA k in slice-major order: slice s meets the weights of kd for output slice d = s - kd
    static constexpr M mfma(int k) {
        int i = 0;
        for (int s = 0; s < 6; ++s)
            for (int kd = 0; kd < 3; ++kd) {
                if (s - kd < 0 || s - kd > 3) continue;
                for (int cb = 0; cb < COB; ++cb) {
                    if (i == k) return M{s, kd, cb};
                    ++i;
                }
            }
        return M{0, 0, 0};
    }
    // slot of fragment read r: spread over the step (the four waves share one LDS port), the slices 3..5
    // first (needed from MFMA 6*COB on), the last one early enough to land before the step ends
    static constexpr int read_slot(int r) { return COB == 2 ? (r < 9 ? 2 * r : 8 + r) : r; }
    // slots of the copies: weight copy 0, weight copy 1, halo copy (address arithmetic in the slots before)
    static constexpr int WC0 = COB == 2 ? 9 : 3, WC1 = COB == 2 ? 11 : 5, HC = COB == 2 ? 15 : 8;
};

template <int COB> struct StepCtx {
    f32x16 (&acc)[COB][4];
    bf16x8 (&acur)[3][COB];
    bf16x8 (&b)[6];
    bf16x8 (&an)[3][COB];
    bf16x8 (&nb)[3];
    const char* hb;          // this step's region + lane offset + tap offset
    const char* hbn;         // the next step's
    const char* wn;          // the next step's weight block + lane offset
    uint32_t wd0, wd1, hd;   // LDS targets of the three copies
    const bf16_t* wb0;       // weight copy sources = wb + woff
    const bf16_t* wb1;
    size_t woff;
    const HaloTile& ht;      // halo copy: tile, this lane's halo coordinates / offset, chunk offset
    int pk, rel, choff;
    const bf16_t* zero16;
    const bf16_t* p0; const bf16_t* p1; const bf16_t* ph; bool in;   // temporaries carried between slots
};

template <int COB, int K>
__device__ __forceinline__ void step_slot(StepCtx<COB>& c) {
    typedef StepPlan<COB> P;
    typedef RW<COB> G;
    constexpr typename P::M m = P::mfma(K);
    c.acc[m.cb][m.s - m.kd] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(c.acur[m.kd][m.cb], c.b[m.s], c.acc[m.cb][m.s - m.kd], 0, 0, 0);
#pragma unroll
    for (int r = 0; r < P::NR; ++r) {
        if (P::read_slot(r) != K) continue;
        if (r < 3) c.b[3 + r] = lds_frag(c.hb + (3 + r) * RSLICE);
        else if (r < 3 + 3 * COB) c.an[(r - 3) / COB][(r - 3) % COB] = lds_frag(c.wn + ((r - 3) / COB) * 2 * G::WPLANE + ((r - 3) % COB) * 512);
        else c.nb[r - 3 - 3 * COB] = lds_frag(c.hbn + (r - 3 - 3 * COB) * RSLICE);
    }
    if constexpr (K == P::WC0 - 1) c.p0 = c.wb0 + c.woff;
    if constexpr (K == P::WC0) g2lds16(c.p0, c.wd0);
    if constexpr (K == P::WC1 - 1) c.p1 = c.wb1 + c.woff;
    if constexpr (K == P::WC1) g2lds16(c.p1, c.wd1);
    if constexpr (K == P::HC - 2) {
        const int hd = c.pk & 255, hh = (c.pk >> 8) & 255, hw = c.pk >> 16;
        c.in = (hd >= c.ht.dlo) & (hd <= c.ht.dhi) & (hh >= c.ht.hlo) & (hh <= c.ht.hhi) & (hw >= c.ht.wlo) & (hw <= c.ht.whi);
    }
    if constexpr (K == P::HC - 1) c.ph = c.in ? c.ht.origin + c.rel + c.choff : c.zero16;
    if constexpr (K == P::HC) g2lds16(c.ph, c.hd);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (K + 1 < P::NM) step_slot<COB, K + 1>(c);
}

// acur / b0..b2: the fragments of this step that were read during the previous one; on return they
// hold the same for the next step.
template <int COB, int J>
__device__ __forceinline__ void ring_step(f32x16 (&acc)[COB][4], bf16x8 (&acur)[3][COB], bf16x8& b0, bf16x8& b1, bf16x8& b2,
                                          const char* hb, const char* hb_nextstep, const char* w_nextstep,
                                          uint32_t w_dst0, uint32_t w_dst1, uint32_t h_dst, const bf16_t* wb0,
                                          const bf16_t* wb1, size_t woff, const HaloTile& ht, int pk, int rel, int choff,
                                          const bf16_t* zero16, bool after_epilogue) {
    constexpr int kh = J / 3, kw = J % 3;
    constexpr int tapoff = (kh * RHW + kw) * 16;
    constexpr int JN = (J + 1) % 9;
    constexpr int tapoff_n = ((JN / 3) * RHW + JN % 3) * 16;
    bf16x8 b[6], an[3][COB], nb[3];
    b[0] = b0; b[1] = b1; b[2] = b2;
    StepCtx<COB> c{acc, acur, b, an, nb, hb + tapoff, hb_nextstep + tapoff_n, w_nextstep, w_dst0, w_dst1, h_dst, wb0, wb1, woff,
                   ht, pk, rel, choff, zero16, nullptr, nullptr, nullptr, false};
    step_slot<COB, 0>(c);
#pragma unroll
    for (int kd = 0; kd < 3; ++kd)
#pragma unroll
        for (int cb = 0; cb < COB; ++cb) acur[kd][cb] = an[kd][cb];
    b0 = nb[0]; b1 = nb[1]; b2 = nb[2];
    // Vector memory operations complete in issue order: leaving RINFLIGHT steps' worth in flight
    // guarantees that everything issued RINFLIGHT or more steps ago has landed -- the weight block two
    // steps ahead (issued 7 steps ago) and every older halo copy.  In the first RINFLIGHT steps after an
    // epilogue the window also holds that epilogue's output stores, which need not be waited for.
    if (after_epilogue) wait_vmcnt<3 * RINFLIGHT + REPI_STORES>();
    else wait_vmcnt<3 * RINFLIGHT>();
    // bare barrier: __syncthreads() would add a release fence that drains every copy in flight
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0), as a builtin so the compiler knows the reads are done
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
}

template <int COB>
__global__ __launch_bounds__(256) void conv3d_ring_kernel(RingArgs a) {
    typedef RW<COB> G;
    constexpr int WROWS = G::WROWS;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char* const hreg = lds;
    char* const wring = lds + RNREG * RREGION;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // in a scalar register: copy targets are wave-uniform
    const int l32 = lane & 31, half = lane >> 5;
    const int co0 = blockIdx.y * WROWS;
    // LDS byte addresses (as the copy instruction wants them) of the two rings
    const uint32_t hreg_a = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)hreg;
    const uint32_t wring_a = hreg_a + RNREG * RREGION;
    const int nchunks = a.Cin >> 4;
    const int spt = nchunks * 9;  // steps per tile

    // persistent walk: the XCD owns a contiguous range of tiles, the workgroup a contiguous run of it
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int tile_lo = xcd * a.tiles_per_xcd + local * a.tiles_per_wg;
    const int tile_hi = min(tile_lo + a.tiles_per_wg, min((xcd + 1) * a.tiles_per_xcd, a.tiles_total));
    if (tile_lo >= tile_hi) return;

    // ---- lane -> voxel of a 32-voxel block (2 h-rows x 16 w).  A 16-byte LDS read is serviced for
    // lanes {0-7,24-31}, {8-15,16-23} (and the same in the upper half) together, so those pairs must
    // fall into opposite 128-byte halves of the bank space: groups of 8 lanes take
    // (row0,w0-7) (row1,w0-7) (row1,w8-15) (row0,w8-15).
    const int g8 = l32 >> 3;
    const int bw = (l32 & 7) + 8 * (g8 >> 1), bh = (g8 ^ (g8 >> 1)) & 1;
    const uint32_t b_base = (uint32_t)(half * RPLANE + ((2 * wv + bh) * RHW + bw) * 16);
    const uint32_t a_base = (uint32_t)(half * G::WPLANE + l32 * 16);

    // ---- per-lane constants of the copies.  Halo copy slot k = J*4 + wv covers entries 60k .. 60k+59 of
    // a region (entry = plane*1080 + halo voxel): rel = element offset from the tile's halo origin.
    int hrel[9], hpk[9], hoff[9];
#pragma unroll
    for (int j = 0; j < 9; ++j) {
        const int e0 = min((j * 4 + wv) * RHSTEP, RHENTRIES - 64);
        const int e = e0 + lane;
        hoff[j] = e0 * 16;
        const int plane = e / RHALO_VOX, hv = e - plane * RHALO_VOX;
        const int hw = hv % RHW, hh = (hv / RHW) % RHH, hd = hv / (RHW * RHH);
        hrel[j] = ((hd * a.H + hh) * a.W + hw) * a.ldx + plane * 8;
        hpk[j] = hd | (hh << 8) | (hw << 16);
    }
    const int we0 = min(wv * G::USTEP, G::WENTRIES - 64), we1 = min((wv + 4) * G::USTEP, G::WENTRIES - 64);
    const bf16_t* wslab0 = a.wp + (size_t)blockIdx.y * 27 * a.Cin * WROWS + (we0 + lane) * 8;
    const bf16_t* wslab1 = a.wp + (size_t)blockIdx.y * 27 * a.Cin * WROWS + (we1 + lane) * 8;

    auto tile_origin = [&](int tile, int& n, int& d0, int& h0, int& w0) {
        n = tile / a.tiles_per_n;
        int r = tile - n * a.tiles_per_n;
        d0 = (r % a.tiles_d) * RTD;
        r /= a.tiles_d;
        w0 = (r % a.tiles_w) * RTW;
        h0 = (r / a.tiles_w) * RTH;
    };
    auto halo_tile = [&](int tile) {
        int n, d0, h0, w0;
        tile_origin(tile, n, d0, h0, w0);
        HaloTile t;
        t.origin = a.x + ((((int64_t)n * a.D + (d0 - 1)) * a.H + (h0 - 1)) * a.W + (w0 - 1)) * a.ldx;
        t.dlo = 1 - d0; t.dhi = a.D - d0; t.hlo = 1 - h0; t.hhi = a.H - h0; t.wlo = 1 - w0; t.whi = a.W - w0;
        return t;
    };
    auto halo_src = [&](const HaloTile& t, int j, int choff) -> const bf16_t* {
        const int pk = hpk[j];
        const int hd = pk & 255, hh = (pk >> 8) & 255, hw = pk >> 16;
        const bool in = (hd >= t.dlo) & (hd <= t.dhi) & (hh >= t.hlo) & (hh <= t.hhi) & (hw >= t.wlo) & (hw <= t.whi);
        return in ? t.origin + hrel[j] + choff : a.zero16;
    };

    // ---- prologue: halo of chunk-steps 0 and 1, weights of steps 0..8
    const int total_q = (tile_hi - tile_lo) * nchunks;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        if (i < total_q) {
            const int t = tile_lo + i / nchunks, c = i % nchunks;
            const HaloTile ht = halo_tile(t);
#pragma unroll
            for (int j = 0; j < 9; ++j) g2lds16(halo_src(ht, j, c * 16), hreg_a + i * RREGION + hoff[j]);
        }
    }
#pragma unroll
    for (int i = 0; i < RNWSLOT; ++i) {
        g2lds16(wslab0 + i * G::WBLOCK_ELEMS, wring_a + i * G::WBLOCK + we0 * 16);
        g2lds16(wslab1 + i * G::WBLOCK_ELEMS, wring_a + i * G::WBLOCK + we1 * 16);
    }
    wait_vmcnt<0>();
    __syncthreads();

    bf16x8 acur[3][COB], b0, b1, b2;
#pragma unroll
    for (int kd = 0; kd < 3; ++kd)
#pragma unroll
        for (int cb = 0; cb < COB; ++cb) acur[kd][cb] = lds_frag(wring + a_base + kd * 2 * G::WPLANE + cb * 512);
    b0 = lds_frag(hreg + b_base);
    b1 = lds_frag(hreg + b_base + RSLICE);
    b2 = lds_frag(hreg + b_base + 2 * RSLICE);

    int rq = 0;                                  // chunk-step counter mod 3: the region being multiplied
    int wsl = 0;                                 // step counter mod 9: the weight slot being multiplied
    int pf_tile = tile_lo + 2 / nchunks, pf_chunk = 2 % nchunks;   // halo prefetch cursor = chunk-step q + 2
    bool epi_full = false;   // the previous tile of the walk lay inside the volume (all its output stores were issued)
    for (int tile = tile_lo; tile < tile_hi; ++tile) {
        f32x16 acc[COB][4];
#pragma unroll
        for (int cb = 0; cb < COB; ++cb)
#pragma unroll
            for (int d = 0; d < 4; ++d)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[cb][d][r] = 0.f;

        for (int chunk = 0; chunk < nchunks; ++chunk) {
            const int rq1 = rq == 2 ? 0 : rq + 1, rq2 = rq == 0 ? 2 : rq - 1;
            const char* hb = hreg + rq * RREGION + b_base;
            const char* hbn = hreg + rq1 * RREGION + b_base;
            // past the end of the walk the copies go on (they keep the in-flight count uniform) and
            // fetch this tile again; nothing reads what they bring
            const uint32_t hdst = hreg_a + rq2 * RREGION;
            const HaloTile ht = halo_tile(pf_tile < tile_hi ? pf_tile : tile);
            const int choff = pf_chunk * 16;
            const int t0 = chunk * 9;
#define RING_STEP(J)                                                                                                  \
    {                                                                                                                 \
        int t9 = t0 + J + RNWSLOT;                                                                                    \
        if (t9 >= spt) t9 -= spt;                                                                                     \
        const int wsl1 = wsl == RNWSLOT - 1 ? 0 : wsl + 1;                                                            \
        const uint32_t wd = wring_a + wsl * G::WBLOCK;                                                                \
        ring_step<COB, J>(acc, acur, b0, b1, b2, hb, (J < 8 ? hb : hbn), wring + wsl1 * G::WBLOCK + a_base,            \
                          wd + we0 * 16, wd + we1 * 16, hdst + hoff[J], wslab0, wslab1, (size_t)t9 * G::WBLOCK_ELEMS,  \
                          ht, hpk[J], hrel[J], choff, a.zero16, J < RINFLIGHT && chunk == 0 && epi_full);             \
        wsl = wsl1;                                                                                                   \
    }
            RING_STEP(0) RING_STEP(1) RING_STEP(2) RING_STEP(3) RING_STEP(4) RING_STEP(5) RING_STEP(6) RING_STEP(7)
            RING_STEP(8)
#undef RING_STEP
            if (++pf_chunk == nchunks) { pf_chunk = 0; ++pf_tile; }
            rq = rq1;
        }

        // ---- epilogue.  Each wave turns its accumulators (lane = voxel, 4 consecutive channels per
        // register group) into voxel rows through a private LDS patch, so that 8 lanes store one full
        // row of 64 channels; the channel sums of the stored values come from the same pass.
        // Scratch: the region of the chunk-step just finished (its refill starts with the next step).
        int n, d0, h0, w0;
        tile_origin(tile, n, d0, h0, w0);
        char* fbuf = hreg + (rq == 0 ? 2 : rq - 1) * RREGION;   // rq was advanced past the last chunk-step
        constexpr int ROWB = WROWS * 2 + 16;           // padded row of the patch
        constexpr int PARTS = WROWS / 8;               // 16-byte parts per row: 8 or 4
        constexpr int RPI = 64 / PARTS;                // rows covered per read instruction
        char* patch = fbuf + wv * (32 * ROWB);
        float* sred = reinterpret_cast<float*>(fbuf + 4 * 32 * (64 * 2 + 16));
        const int part = lane % PARTS, prow = lane / PARTS;
        float csum[8], csq[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { csum[e] = 0.f; csq[e] = 0.f; }
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int gd = d0 + d;
#pragma unroll
            for (int cb = 0; cb < COB; ++cb)
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    const uint32_t p0 = pack_bf16(acc[cb][d][rg * 4 + 0], acc[cb][d][rg * 4 + 1]);
                    const uint32_t p1 = pack_bf16(acc[cb][d][rg * 4 + 2], acc[cb][d][rg * 4 + 3]);
                    *reinterpret_cast<uint2*>(patch + l32 * ROWB + (cb * 32 + rg * 8 + half * 4) * 2) = make_uint2(p0, p1);
                }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int i = 0; i < 32 / RPI; ++i) {
                const int row = prow + i * RPI;          // voxel index inside the 32-voxel block
                const uint4 qv = *reinterpret_cast<const uint4*>(patch + row * ROWB + part * 16);
                const int rg8 = row >> 3;
                const int rw = (row & 7) + 8 * (rg8 >> 1), rh = (rg8 ^ (rg8 >> 1)) & 1;
                const int gh = h0 + 2 * wv + rh, gw = w0 + rw;
                const bool ok = gd < a.D && gh < a.H && gw < a.W;
                if (ok) {
                    // streaming store: the output is not read again by this kernel and should not displace the
                    // input lines that the next chunk passes and the neighbouring tiles still need
                    typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
                    const u32x4 sv = {qv.x, qv.y, qv.z, qv.w};
                    __builtin_nontemporal_store(
                        sv, reinterpret_cast<u32x4*>(a.z + ((((int64_t)n * a.D + gd) * a.H + gh) * a.W + gw) * a.ldz + co0 + part * 8));
                    const uint32_t r4[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float f0 = __uint_as_float(r4[e] << 16), f1 = __uint_as_float(r4[e] & 0xFFFF0000u);
                        csum[2 * e] += f0; csq[2 * e] = fmaf(f0, f0, csq[2 * e]);
                        csum[2 * e + 1] += f1; csq[2 * e + 1] = fmaf(f1, f1, csq[2 * e + 1]);
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
        if (a.part) {
            // lanes with equal `part` hold the same 8 channels: fold them (lane bits above log2(PARTS))
#pragma unroll
            for (int e = 0; e < 8; ++e) {
#pragma unroll
                for (int m = PARTS; m < 64; m <<= 1) {
                    csum[e] += __shfl_xor(csum[e], m);
                    csq[e] += __shfl_xor(csq[e], m);
                }
            }
            if (lane < PARTS) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    sred[(wv * 64 + part * 8 + e) * 2 + 0] = csum[e];
                    sred[(wv * 64 + part * 8 + e) * 2 + 1] = csq[e];
                }
            }
            __builtin_amdgcn_s_waitcnt(0xC07F);  // LDS writes done; a bare barrier leaves the output stores in flight
            __builtin_amdgcn_s_barrier();
            if (tid < WROWS * 2) {
                const int c = tid >> 1, k = tid & 1;
                float v = 0.f;
#pragma unroll
                for (int w4 = 0; w4 < 4; ++w4) v += sred[(w4 * 64 + c) * 2 + k];
                a.part[(((int64_t)n * a.tiles_per_n + (tile - n * a.tiles_per_n)) * a.Cout + co0 + c) * 2 + k] = v;
            }
            if (a.counts && tid == 0 && n == 0 && blockIdx.y == 0)
                a.counts[tile] = min(RTD, a.D - d0) * min(RTH, a.H - h0) * min(RTW, a.W - w0);
        }
        // the patch region is the next step's prefetch target (bare barrier: the output stores stay in flight)
        __builtin_amdgcn_s_waitcnt(0xC07F);
        __builtin_amdgcn_s_barrier();
        epi_full = d0 + RTD <= a.D && h0 + RTH <= a.H && w0 + RTW <= a.W;
    }
    wait_vmcnt<0>();  // the last steps' copies may still be in flight
}

template <int COB>
lamp_status launch_ring(const RingArgs& a, dim3 grid, hipStream_t s) {
    static bool attr_done = false;
    const int shm = RW<COB>::LDS_BYTES;
    if (!attr_done) {
        if (hipFuncSetAttribute((const void*)conv3d_ring_kernel<COB>, hipFuncAttributeMaxDynamicSharedMemorySize, shm) != hipSuccess)
            return LAMP_ERR_HIP;
        attr_done = true;
    }
    hipLaunchKernelGGL((conv3d_ring_kernel<COB>), grid, dim3(256), shm, s, a);
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}

}  // namespace

lamp_status ring_conv_fwd(const lamp_tensor_desc* xd, const void* x, const void* w, bool dgrad, const lamp_tensor_desc* zd,
                          void* z, float* stats_out, float eps, void* ws, size_t ws_bytes, hipStream_t s) {
    if ((((uintptr_t)x) & 15u) || (((uintptr_t)z) & 15u) || (((uintptr_t)ws) & 15u)) return LAMP_ERR_ALIGN;
    const int td = (zd->d + RTD - 1) / RTD, th = (zd->h + RTH - 1) / RTH, tw = (zd->w + RTW - 1) / RTW;
    const int tiles_per_n = td * th * tw;
    Carver cv(ws, ws_bytes);
    bf16_t* wp = (bf16_t*)cv.take((size_t)27 * xd->c * zd->c * 2 + 16);
    float* part = nullptr;
    int32_t* counts = nullptr;
    if (stats_out) {
        part = (float*)cv.take((size_t)zd->n * tiles_per_n * zd->c * 2 * sizeof(float));
        counts = (int32_t*)cv.take((size_t)tiles_per_n * sizeof(int32_t));
    }
    if (!cv.ok()) return LAMP_ERR_WORKSPACE;
    const int cob = (zd->c % 64 == 0) ? 2 : 1;
    const int64_t wtotal = (int64_t)27 * xd->c * zd->c;
    hipLaunchKernelGGL(ring_repack_kernel, dim3(cdiv(wtotal, 256)), dim3(256), 0, s, (const bf16_t*)w, wp, zd->c, xd->c,
                       32 * cob, dgrad ? 1 : 0);
    LAMP_CHECK_LAUNCH();
    RingArgs a;
    a.x = (const bf16_t*)x; a.ldx = xd->ldc; a.wp = wp; a.z = (bf16_t*)z; a.ldz = zd->ldc; a.part = part; a.counts = counts;
    a.zero16 = wp + (size_t)27 * xd->c * zd->c;
    a.N = zd->n; a.D = zd->d; a.H = zd->h; a.W = zd->w; a.Cin = xd->c; a.Cout = zd->c;
    a.tiles_d = td; a.tiles_h = th; a.tiles_w = tw; a.tiles_per_n = tiles_per_n;
    a.tiles_total = tiles_per_n * zd->n;
    a.tiles_per_xcd = (a.tiles_total + 7) / 8;
    int wg_per_xcd = a.tiles_per_xcd < 32 ? a.tiles_per_xcd : 32;  // one persistent workgroup per CU (LDS-limited)
    a.tiles_per_wg = (a.tiles_per_xcd + wg_per_xcd - 1) / wg_per_xcd;
    wg_per_xcd = (a.tiles_per_xcd + a.tiles_per_wg - 1) / a.tiles_per_wg;
    dim3 grid(8 * wg_per_xcd, zd->c / (32 * cob));
    lamp_status st = cob == 2 ? launch_ring<2>(a, grid, s) : launch_ring<1>(a, grid, s);
    if (st != LAMP_OK) return st;
    if (stats_out) return launch_stats_finalize(part, counts, tiles_per_n, zd->n, zd->c, eps, stats_out, s);
    return LAMP_OK;
}

}  // namespace lamp
