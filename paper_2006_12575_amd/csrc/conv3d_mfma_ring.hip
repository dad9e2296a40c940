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
//  * LDS holds a ring of 3 halo regions, each one 16-channel chunk of a tile's 6 x 10 x 18 halo (32 bytes
//    per voxel, fetched as one request), and a ring of 8 weight blocks (3 taps x 16 ci x 32*COB co).
//    Region (q+2)%3 is refilled for chunk-step q+2 while chunk-step q is multiplied, weight block s%8
//    for step s+8 while step s is multiplied, both by register-free global -> LDS copies.  Copies
//    complete in issue order, so the long weight ring is what lets a halo copy that misses every
//    cache stay in flight for 6 steps without holding up the weights behind it.
//  * One step = one (chunk, kh, kw); a barrier per step publishes the copies two steps ahead of their
//    use, so fragment reads for step s+1 are issued inside step s and the MFMA stream never drains.
//  * With one wave per SIMD nothing runs while a wave converts and stores its results, so the epilogue
//    of a tile is cut into small units (convert + write to a private LDS patch; read a voxel row back,
//    store it, add it to the channel sums) that ride in the steps of the NEXT tile, which accumulates
//    into a second set of registers.
//  * Tiles are numbered d-fastest, an XCD owns a contiguous range of them and its persistent workgroups
//    take them in turn: at any time the workgroups of an XCD work on neighbouring tiles (a column in d
//    first), whose shared halo voxels are then fetched from memory once and re-read from the XCD's L2.
#include <stdlib.h>
#include <type_traits>
#include "internal.h"
#include "repack.h"

namespace lamp {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int RTD = 4, RTH = 8, RTW = 16;
constexpr int RHD = RTD + 2, RHH = RTH + 2, RHW = RTW + 2;
constexpr int RHALO_VOX = RHD * RHH * RHW;   // 1080
constexpr int RREGION = RHALO_VOX * 32;      // one 16-channel chunk (32 bytes per voxel): 34560
constexpr int RNREG = 3;
constexpr int RSLICE = RHH * RHW * 32;       // bytes between halo d-slices
constexpr int RROW = RHW * 32;               // bytes between halo h-rows
constexpr int RHENTRIES = 2 * RHALO_VOX;     // 16-byte entries of a region: 36 wave copies, 9 per wave, copy k
constexpr int RHSTEP = 60;                   // starts at entry min(60k, 2160-64) (neighbours overlap by 4 entries)
constexpr int RNWSLOT = 8;                  // weight ring: block of step s + 8 replaces block s
constexpr int RINFLIGHT = 6;                // steps whose copies may still be in flight at a step's end
constexpr int RPATCH_ROW = 80;              // epilogue patch row: 32 channels (64 bytes) + 16 bytes of padding
constexpr int RPATCH = 32 * RPATCH_ROW;     // one wave's patch: the 32 voxels of a block

template <int COB> struct RW {
    static constexpr int WROWS = 32 * COB;
    static constexpr int WPLANE = WROWS * 16;        // one (tap, plane): WROWS rows of 16 bytes
    static constexpr int WBLOCK = 6 * WPLANE;        // 3 taps (kd) x 2 planes
    static constexpr int WBLOCK_ELEMS = WBLOCK / 2;
    static constexpr int WENTRIES = 6 * WROWS;       // 16-byte entries of a block: 8 wave copies, 2 per wave, copy u
    static constexpr int USTEP = WENTRIES / 8;       // starts at entry min(u * USTEP, WENTRIES - 64)
    static constexpr int LDS_BYTES = RNREG * RREGION + RNWSLOT * WBLOCK + 4 * RPATCH;
};

struct RingArgs {
    const bf16_t* x; int ldx;
    const bf16_t* wp;
    bf16_t* z; int ldz;
    float* part;           // [N][4 * workgroups][Cout][2]: per-wave partial (sum, sum of squares), or nullptr
    int32_t* counts;       // [N][4 * workgroups]: voxels behind each partial (written when part != nullptr)
    const bf16_t* zero16;  // 2 * Cin + 16 zero bytes in global memory (source of the zero padding, any chunk offset)
    bf16_t* dump;          // 16 bytes in global memory that absorb the stores of voxels outside the volume
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
    repack_ring_gran(w, wp, (int64_t)blockIdx.x * 256 + threadIdx.x, Cout, Cin, wrows, dgrad);
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

// ---- epilogue of the previous ("pending") tile.  Its results, converted to bf16 pairs when the tile
// ended, sit in a second register set `pend` (lane = voxel of a 32-voxel block, 4 consecutive channels
// = 2 registers per register group).  The epilogue runs in 2*COB phases, one per chunk-step: phase p
// handles channel block p / 2 and d-slices 2 * (p % 2), 2 * (p % 2) + 1, three steps each:
//   unit A(rg), rg = 0..3 : write 4 channels to the wave's LDS patch (32 voxel rows of 64 bytes)
//   unit B(i),  i = 0..1  : 4 lanes read back one voxel row (16 rows per instruction), store its 64 bytes
//                           and add the stored values to this lane's channel sums
// There is one copy of the code for all phases: they all take their data from `front`, which is
// reloaded from `pend` after every phase, and the channel sums of the two blocks swap places when the
// block changes.  Voxels outside the volume are zeroed when the tile ends, so they add nothing to the
// sums; their rows are stored to a dump address.  With nothing pending the units still run, on zeros.
// The channel sums run on across the tiles of the walk and are written once per sample.
template <int COB> struct EpiCtx {
    uint32_t (&front)[2][8];
    float (&csum)[8];
    float (&csq)[8];
    char* patch_w;        // patch + l32 * RPATCH_ROW + half * 8      (unit A adds rg * 16)
    const char* patch_r;  // patch + (lane / 4) * RPATCH_ROW + (lane % 4) * 16   (unit B adds i * 16 rows)
    bf16_t* zp[2];        // output address of this lane's row of group i in d-slice 0, channel block 0
    bool okl[2];          // that row's (h, w) lies inside the volume (and a phase is in progress)
    int64_t dstride;      // elements between d-slices of the output
    int64_t poff;         // element offset of the phase: first d-slice and channel block
    int dleft;            // d-slices inside the volume, counted from the phase's first
    bf16_t* dump;
    uint4 q;              // row in flight between the slots of a unit B
    bf16_t* qp;
};

template <int COB, int DD, int RG>
__device__ __forceinline__ void epi_unit_a(EpiCtx<COB>& e) {
    *reinterpret_cast<uint2*>(e.patch_w + RG * 16) = make_uint2(e.front[DD][RG * 2], e.front[DD][RG * 2 + 1]);
}
template <int COB, int I> __device__ __forceinline__ void epi_unit_b_read(EpiCtx<COB>& e) {
    e.q = *reinterpret_cast<const uint4*>(e.patch_r + I * 16 * RPATCH_ROW);
}
template <int COB, int DD, int I> __device__ __forceinline__ void epi_unit_b_addr(EpiCtx<COB>& e) {
    const bool ok = e.okl[I] & (DD < e.dleft);
    e.qp = ok ? e.zp[I] + (e.poff + DD * e.dstride) : e.dump;
}
template <int COB, int DD, int I> __device__ __forceinline__ void epi_unit_b_store(EpiCtx<COB>& e) {
    // streaming store: the output is not read again by this kernel and should not displace the input
    // lines that the next chunk passes and the neighbouring tiles still need
    typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
    const u32x4 sv = {e.q.x, e.q.y, e.q.z, e.q.w};
    __builtin_nontemporal_store(sv, reinterpret_cast<u32x4*>(e.qp));
}
template <int COB, int E> __device__ __forceinline__ void epi_unit_b_stats(EpiCtx<COB>& e) {
    const uint32_t r = E == 0 ? e.q.x : E == 1 ? e.q.y : E == 2 ? e.q.z : e.q.w;
    const float f0 = __uint_as_float(r << 16), f1 = __uint_as_float(r & 0xFFFF0000u);
    e.csum[2 * E] += f0;
    e.csq[2 * E] = fmaf(f0, f0, e.csq[2 * E]);
    e.csum[2 * E + 1] += f1;
    e.csq[2 * E + 1] = fmaf(f1, f1, e.csq[2 * E + 1]);
}
// A whole phase in one go (used where no step is left to carry the units).
template <int COB> __device__ __forceinline__ void epi_phase_serial(EpiCtx<COB>& e) {
    auto one_d = [&](auto dt) __attribute__((always_inline)) {
        constexpr int DD = decltype(dt)::value;
        epi_unit_a<COB, DD, 0>(e); epi_unit_a<COB, DD, 1>(e); epi_unit_a<COB, DD, 2>(e); epi_unit_a<COB, DD, 3>(e);
        epi_unit_b_read<COB, 0>(e); epi_unit_b_addr<COB, DD, 0>(e); epi_unit_b_store<COB, DD, 0>(e);
        epi_unit_b_stats<COB, 0>(e); epi_unit_b_stats<COB, 1>(e); epi_unit_b_stats<COB, 2>(e); epi_unit_b_stats<COB, 3>(e);
        epi_unit_b_read<COB, 1>(e); epi_unit_b_addr<COB, DD, 1>(e); epi_unit_b_store<COB, DD, 1>(e);
        epi_unit_b_stats<COB, 0>(e); epi_unit_b_stats<COB, 1>(e); epi_unit_b_stats<COB, 2>(e); epi_unit_b_stats<COB, 3>(e);
    };
    one_d(std::integral_constant<int, 0>{});
    one_d(std::integral_constant<int, 1>{});
}
// The share of slot K of step J: steps 0..2 carry unit A x 4, unit B(0), unit B(1) of the phase's first
// d-slice, steps 3..5 those of its second.
template <int COB, int J, int K>
__device__ __forceinline__ void epi_slot(EpiCtx<COB>& e) {
    if constexpr (J < 6) {
        constexpr int DD = J / 3, PH = J % 3;
        constexpr int S = COB == 2 ? 2 : 1;   // slot stride: the step has 24 or 12 slots
        if constexpr (PH == 0) {
            if constexpr (K == 1 * S) epi_unit_a<COB, DD, 0>(e);
            if constexpr (K == 3 * S) epi_unit_a<COB, DD, 1>(e);
            if constexpr (K == 5 * S) epi_unit_a<COB, DD, 2>(e);
            if constexpr (K == 7 * S) epi_unit_a<COB, DD, 3>(e);
        } else {
            constexpr int I = PH - 1;
            if constexpr (K == 0) epi_unit_b_read<COB, I>(e);
            if constexpr (K == 1 * S) epi_unit_b_addr<COB, DD, I>(e);
            if constexpr (K == 3 * S) epi_unit_b_store<COB, DD, I>(e);
            if constexpr (K == 4 * S) epi_unit_b_stats<COB, 0>(e);
            if constexpr (K == 5 * S) epi_unit_b_stats<COB, 1>(e);
            if constexpr (K == 8 * S) epi_unit_b_stats<COB, 2>(e);
            if constexpr (K == 9 * S) epi_unit_b_stats<COB, 3>(e);
        }
    }
}

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
    const HaloTile& ht;      // halo copy: tile, this lane's halo coordinates (pk = hd | hh << 8 | hw << 16 |
    int pk, choff;           //   plane << 24), chunk offset; hptr = source address for chunk 0, kept per tile
    int H, W, ldx;
    const bf16_t* zeros;
    const bf16_t*& hptr;
    bool newtile;            // hptr must be computed (the prefetched tile changed)
    const bf16_t* p0; const bf16_t* p1; bool in;   // temporaries carried between slots
};

template <int COB, int J, int K>
__device__ __forceinline__ void step_slot(StepCtx<COB>& c, EpiCtx<COB>& e) {
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
    // the halo source of this lane changes only with the prefetched tile: voxels outside the volume read
    // from a run of zeros that is long enough for every chunk offset
    if constexpr (K == P::HC - 2) {
        if (c.newtile) {
            const int hd = c.pk & 255, hh = (c.pk >> 8) & 255, hw = (c.pk >> 16) & 255;
            c.in = (hd >= c.ht.dlo) & (hd <= c.ht.dhi) & (hh >= c.ht.hlo) & (hh <= c.ht.hhi) & (hw >= c.ht.wlo) & (hw <= c.ht.whi);
        }
    }
    if constexpr (K == P::HC - 1) {
        if (c.newtile) {
            const int hd = c.pk & 255, hh = (c.pk >> 8) & 255, hw = (c.pk >> 16) & 255, plane = c.pk >> 24;
            c.hptr = c.in ? c.ht.origin + (((hd * c.H + hh) * c.W + hw) * c.ldx + plane * 8) : c.zeros;
        }
    }
    if constexpr (K == P::HC) g2lds16(c.hptr + c.choff, c.hd);
    epi_slot<COB, J, K>(e);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (K + 1 < P::NM) step_slot<COB, J, K + 1>(c, e);
}

// acur / b0..b2: the fragments of this step that were read during the previous one; on return they
// hold the same for the next step.
template <int COB, int J>
__device__ __forceinline__ void ring_step(f32x16 (&acc)[COB][4], bf16x8 (&acur)[3][COB], bf16x8& b0, bf16x8& b1, bf16x8& b2,
                                          const char* hr, const char* hr_nextstep, const uint32_t (&bb)[3],
                                          const char* w_nextstep,
                                          uint32_t w_dst0, uint32_t w_dst1, uint32_t h_dst, const bf16_t* wb0,
                                          const bf16_t* wb1, size_t woff, const HaloTile& ht, int pk, int choff, int H,
                                          int W, int ldx, const bf16_t* zeros, const bf16_t*& hptr, bool newtile,
                                          EpiCtx<COB>& e) {
    constexpr int kh = J / 3, kw = J % 3;
    constexpr int JN = (J + 1) % 9;
    constexpr int khn = JN / 3, kwn = JN % 3;
    bf16x8 b[6], an[3][COB], nb[3];
    b[0] = b0; b[1] = b1; b[2] = b2;
    StepCtx<COB> c{acc, acur, b, an, nb, hr + (bb[kw] + kh * RROW), hr_nextstep + (bb[kwn] + khn * RROW), w_nextstep, w_dst0, w_dst1, h_dst, wb0, wb1, woff,
                   ht, pk, choff, H, W, ldx, zeros, hptr, newtile, nullptr, nullptr, false};
    step_slot<COB, J, 0>(c, e);
#pragma unroll
    for (int kd = 0; kd < 3; ++kd)
#pragma unroll
        for (int cb = 0; cb < COB; ++cb) acur[kd][cb] = an[kd][cb];
    b0 = nb[0]; b1 = nb[1]; b2 = nb[2];
    // Vector memory operations complete in issue order: leaving the copies of RINFLIGHT steps in flight
    // guarantees that everything issued RINFLIGHT or more steps ago has landed -- the weight block two
    // steps ahead (issued 6 steps ago) and every older halo copy.  (Output stores issued in between only
    // make the wait reach further back.)
    wait_vmcnt<3 * RINFLIGHT>();
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
    const int tstep = (int)(gridDim.x >> 3);   // the workgroups of an XCD take its tiles in turn, so that at any
    const int tile_lo = xcd * a.tiles_per_xcd + local;   // time they work on neighbours (in d first) and share halos in L2
    const int tile_hi = min((xcd + 1) * a.tiles_per_xcd, a.tiles_total);
    // voxel counts behind this wave's partial statistics: zero for the samples it never visits
    if (a.counts && lane == 0 && blockIdx.y == 0)
        for (int n = 0; n < a.N; ++n) a.counts[n * (gridDim.x * 4) + blockIdx.x * 4 + wv] = 0;
    if (tile_lo >= tile_hi) return;

    // ---- lane -> voxel of a 32-voxel block (2 h-rows x 16 w).  A 16-byte LDS read is serviced for
    // lanes {0-7,24-31}, {8-15,16-23} (and the same in the upper half) together, so those pairs must
    // fall into opposite 128-byte halves of the bank space: groups of 8 lanes take
    // (row0,w0-7) (row1,w0-7) (row1,w8-15) (row0,w8-15).
    const int g8 = l32 >> 3;
    const int bw = (l32 & 7) + 8 * (g8 >> 1), bh = (g8 ^ (g8 >> 1)) & 1;
    // A region holds, per halo voxel, the 32 bytes of the chunk as two 16-byte halves (channels 0-7 / 8-15),
    // swapped for voxels whose w coordinate has bit 3 set: the two lanes of a copy that fetch one voxel
    // are neighbours (one 32-byte request), and a fragment read -- 16 consecutive w per row, one half --
    // still spreads over all banks.  bb[kw]: this lane's read offset for the in-plane tap column kw.
    uint32_t bb[3];
#pragma unroll
    for (int kw = 0; kw < 3; ++kw)
        bb[kw] = (uint32_t)((((2 * wv + bh) * RHW + bw + kw) * 32) + ((half ^ (((bw + kw) >> 3) & 1)) * 16));
    const uint32_t a_base = (uint32_t)(half * G::WPLANE + l32 * 16);

    // ---- per-lane constants of the copies.  Halo copy slot k = J*4 + wv covers the 16-byte entries
    // 60k .. 60k+63 of a region (entry = 2 * halo voxel + half).
    int hpk[9], hoff[9];   // hd | hh << 8 | hw << 16 | plane << 24 of this lane's entry; LDS offset of the copy
#pragma unroll
    for (int j = 0; j < 9; ++j) {
        const int e0 = min((j * 4 + wv) * RHSTEP, RHENTRIES - 64);
        const int e = e0 + lane;
        hoff[j] = e0 * 16;
        const int hv = e >> 1;
        const int hw = hv % RHW, hh = (hv / RHW) % RHH, hd = hv / (RHW * RHH);
        const int plane = (e & 1) ^ ((hw >> 3) & 1);   // which 8 channels of the chunk this entry holds
        hpk[j] = hd | (hh << 8) | (hw << 16) | (plane << 24);
    }
    const int we0 = min(wv * G::USTEP, G::WENTRIES - 64), we1 = min((wv + 4) * G::USTEP, G::WENTRIES - 64);
    const bf16_t* wslab0 = a.wp + (size_t)blockIdx.y * 27 * a.Cin * WROWS + (we0 + lane) * 8;
    const bf16_t* wslab1 = a.wp + (size_t)blockIdx.y * 27 * a.Cin * WROWS + (we1 + lane) * 8;

    auto tile_origin = [&](int tile, int& n, int& d0, int& h0, int& w0) __attribute__((always_inline)) {
        n = tile / a.tiles_per_n;
        int r = tile - n * a.tiles_per_n;
        d0 = (r % a.tiles_d) * RTD;
        r /= a.tiles_d;
        w0 = (r % a.tiles_w) * RTW;
        h0 = (r / a.tiles_w) * RTH;
    };
    auto halo_tile = [&](int tile) __attribute__((always_inline)) {
        int n, d0, h0, w0;
        tile_origin(tile, n, d0, h0, w0);
        HaloTile t;
        t.origin = a.x + ((((int64_t)n * a.D + (d0 - 1)) * a.H + (h0 - 1)) * a.W + (w0 - 1)) * a.ldx;
        t.dlo = 1 - d0; t.dhi = a.D - d0; t.hlo = 1 - h0; t.hhi = a.H - h0; t.wlo = 1 - w0; t.whi = a.W - w0;
        return t;
    };
    auto halo_src = [&](const HaloTile& t, int j, int choff) -> const bf16_t* {
        const int pk = hpk[j];
        const int hd = pk & 255, hh = (pk >> 8) & 255, hw = (pk >> 16) & 255, plane = pk >> 24;
        const bool in = (hd >= t.dlo) & (hd <= t.dhi) & (hh >= t.hlo) & (hh <= t.hhi) & (hw >= t.wlo) & (hw <= t.whi);
        return in ? t.origin + (((hd * a.H + hh) * a.W + hw) * a.ldx + plane * 8 + choff) : a.zero16;
    };

    // ---- prologue: halo of chunk-steps 0 and 1, weights of steps 0..8
    const int total_q = ((tile_hi - tile_lo + tstep - 1) / tstep) * nchunks;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        if (i < total_q) {
            const int t = tile_lo + (i / nchunks) * tstep, c = i % nchunks;
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
    b0 = lds_frag(hreg + bb[0]);
    b1 = lds_frag(hreg + bb[0] + RSLICE);
    b2 = lds_frag(hreg + bb[0] + 2 * RSLICE);

    int rq = 0;                                  // chunk-step counter mod 3: the region being multiplied
    int wsl = 0;                                 // step counter mod 8: the weight slot being multiplied
    int pf_tile = tile_lo + (2 / nchunks) * tstep, pf_chunk = 2 % nchunks;   // halo prefetch cursor = chunk-step q + 2

    // ---- the pending tile: results of the previous tile of the walk, on their way out
    constexpr int NPH = 2 * COB;
    f32x16 acc[COB][4];
    uint32_t front[2][8];            // data of the phase in progress: [dd] = d-slice 2 * dp + dd of block cb
    uint32_t pend[NPH - 1][2][8];    // data of the phases 1 .. NPH-1 (phase p = cb * 2 + dp)
    const bf16_t* hptr[9];           // halo copy sources of the prefetched tile (chunk 0), one per step
    int hptr_tile = -1;              // the tile they belong to
    float csum[8], csq[8];           // channel sums of the block in progress ...
    float osum[8], osq[8];           // ... and of the other block (COB == 2)
    char* const patch = lds + RNREG * RREGION + RNWSLOT * G::WBLOCK + wv * RPATCH;
    EpiCtx<COB> ec{front, csum, csq, patch + l32 * RPATCH_ROW + half * 8, patch + (lane >> 2) * RPATCH_ROW + (lane & 3) * 16,
                   {a.dump, a.dump}, {false, false}, (int64_t)a.H * a.W * a.ldz, 0, 0, a.dump, make_uint4(0, 0, 0, 0), a.dump};
    bool okt[2] = {false, false};   // (h, w) of this lane's two rows of the pending tile lie inside the volume
    int dvalid = 0;                  // d-slices of the pending tile inside the volume
    int epi_p = NPH;                 // next phase of the pending tile to go out (NPH: nothing pending)
    int stat_n = -1;                 // sample the running channel sums belong to
    int stat_vox = 0;                // voxels (of this wave) in them
    const int spart = blockIdx.x * 4 + wv, sparts = gridDim.x * 4;   // this wave's slot in the partial statistics

    // set the context up for phase epi_p
    auto phase_setup = [&]() __attribute__((always_inline)) {
        const bool act = epi_p < NPH;
        const int cb = epi_p >> 1, dp = epi_p & 1;
        ec.okl[0] = okt[0] && act;
        ec.okl[1] = okt[1] && act;
        ec.poff = (int64_t)(2 * dp) * ec.dstride + cb * 32;
        ec.dleft = dvalid - 2 * dp;
    };
    // a phase is done: bring the next one's data to the front (zeros when nothing is left)
    auto phase_advance = [&]() __attribute__((always_inline)) {
        if (epi_p < NPH) {
            const int np = epi_p + 1;
#pragma unroll
            for (int dd = 0; dd < 2; ++dd)
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    uint32_t v = 0u;
                    if (np == 1) v = pend[0][dd][r];
                    if (COB == 2 && np == 2) v = pend[NPH > 2 ? 1 : 0][dd][r];
                    if (COB == 2 && np == 3) v = pend[NPH > 3 ? 2 : 0][dd][r];
                    front[dd][r] = v;
                }
            if (COB == 2 && (epi_p & 1)) {   // the channel block changes
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float t0 = csum[e], t1 = csq[e];
                    csum[e] = osum[e]; csq[e] = osq[e];
                    osum[e] = t0; osq[e] = t1;
                }
            }
            ++epi_p;
        }
        phase_setup();
    };
    // Flush what is left of the pending tile.
    auto finish_pending = [&]() __attribute__((always_inline)) {
        while (epi_p < NPH) {
            epi_phase_serial<COB>(ec);
            phase_advance();
        }
    };
    // Write the running channel sums as this wave's partial statistics of sample stat_n and clear them.
    // (Called between tiles only: csum/csq then hold block 0 and osum/osq block 1.)
    auto flush_stats = [&]() __attribute__((always_inline)) {
        if (a.part && stat_n >= 0) {
            // lanes with equal lane % 4 hold the same 8 channels of a block: fold the other lane bits
#pragma unroll
            for (int e = 0; e < 8; ++e)
#pragma unroll
                for (int m = 4; m < 64; m <<= 1) {
                    csum[e] += __shfl_xor(csum[e], m);
                    csq[e] += __shfl_xor(csq[e], m);
                    if (COB == 2) {
                        osum[e] += __shfl_xor(osum[e], m);
                        osq[e] += __shfl_xor(osq[e], m);
                    }
                }
            if (lane < 4) {
                float* pp = a.part + (((int64_t)stat_n * sparts + spart) * a.Cout + co0 + lane * 8) * 2;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    pp[e * 2 + 0] = csum[e];
                    pp[e * 2 + 1] = csq[e];
                    if (COB == 2) {
                        pp[(32 + e) * 2 + 0] = osum[e];
                        pp[(32 + e) * 2 + 1] = osq[e];
                    }
                }
            }
            if (lane == 0 && blockIdx.y == 0) a.counts[stat_n * sparts + spart] = stat_vox;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) { csum[e] = 0.f; csq[e] = 0.f; osum[e] = 0.f; osq[e] = 0.f; }
        stat_vox = 0;
    };

#pragma unroll
    for (int e = 0; e < 8; ++e) { csum[e] = 0.f; csq[e] = 0.f; osum[e] = 0.f; osq[e] = 0.f; }
#pragma unroll
    for (int dd = 0; dd < 2; ++dd)
#pragma unroll
        for (int r = 0; r < 8; ++r) front[dd][r] = 0u;
#pragma unroll
    for (int cb = 0; cb < COB; ++cb)
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[cb][d][r] = 0.f;
    phase_setup();

    for (int tile = tile_lo; tile < tile_hi; tile += tstep) {
        for (int chunk = 0; chunk < nchunks; ++chunk) {
            const int rq1 = rq == 2 ? 0 : rq + 1, rq2 = rq == 0 ? 2 : rq - 1;
            const char* hr = hreg + rq * RREGION;
            const char* hrn = hreg + rq1 * RREGION;
            // past the end of the walk the copies go on (they keep the in-flight count uniform) and
            // fetch this tile again; nothing reads what they bring
            const uint32_t hdst = hreg_a + rq2 * RREGION;
            const int src_tile = pf_tile < tile_hi ? pf_tile : tile;
            const HaloTile ht = halo_tile(src_tile);
            const bool newtile = src_tile != hptr_tile;
            hptr_tile = src_tile;
            const int choff = pf_chunk * 16;
            const int t0 = chunk * 9;
#define RING_STEP(J)                                                                                                  \
    {                                                                                                                 \
        int t8 = t0 + J + RNWSLOT;                                                                                    \
        if (t8 >= spt) t8 -= spt;                                                                                     \
        const int wsl1 = wsl == RNWSLOT - 1 ? 0 : wsl + 1;                                                            \
        const uint32_t wd = wring_a + wsl * G::WBLOCK;                                                                \
        ring_step<COB, J>(acc, acur, b0, b1, b2, hr, (J < 8 ? hr : hrn), bb, wring + wsl1 * G::WBLOCK + a_base,        \
                          wd + we0 * 16, wd + we1 * 16, hdst + hoff[J], wslab0, wslab1, (size_t)t8 * G::WBLOCK_ELEMS,  \
                          ht, hpk[J], choff, a.H, a.W, a.ldx, a.zero16, hptr[J], newtile, ec);                         \
        wsl = wsl1;                                                                                                   \
    }
            RING_STEP(0) RING_STEP(1) RING_STEP(2) RING_STEP(3) RING_STEP(4) RING_STEP(5) RING_STEP(6) RING_STEP(7)
            RING_STEP(8)
#undef RING_STEP
            phase_advance();
            if (++pf_chunk == nchunks) { pf_chunk = 0; pf_tile += tstep; }
            rq = rq1;
        }

        // ---- tile end: the previous tile must be out before this one takes its place
        finish_pending();
        int n, d0, h0, w0;
        tile_origin(tile, n, d0, h0, w0);
        if (n != stat_n) { flush_stats(); stat_n = n; }
        dvalid = min(RTD, a.D - d0);
        // this lane's voxel of the blocks (as the MFMA result holds them): inside the volume in h and w?
        const bool hw_in = h0 + 2 * wv + bh < a.H && w0 + bw < a.W;
#pragma unroll
        for (int cb = 0; cb < COB; ++cb)
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const uint32_t keep = (hw_in && d < dvalid) ? 0xFFFFFFFFu : 0u;   // voxels outside the volume become zeros
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    const uint32_t v = pack_bf16(acc[cb][d][2 * r], acc[cb][d][2 * r + 1]) & keep;
                    if (cb == 0 && d < 2) front[d][r] = v;
                    else pend[cb * 2 + (d >> 1) - 1][d & 1][r] = v;
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[cb][d][r] = 0.f;
            }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = (lane >> 2) + 16 * i;   // voxel index inside the 32-voxel block
            const int rg8 = row >> 3;
            const int rw = (row & 7) + 8 * (rg8 >> 1), rh = (rg8 ^ (rg8 >> 1)) & 1;
            const int gh = h0 + 2 * wv + rh, gw = w0 + rw;
            okt[i] = gh < a.H && gw < a.W;
            ec.zp[i] = a.z + ((((int64_t)n * a.D + d0) * a.H + gh) * a.W + gw) * a.ldz + co0 + (lane & 3) * 8;
        }
        stat_vox += dvalid * max(0, min(2, a.H - (h0 + 2 * wv))) * min(RTW, a.W - w0);
        epi_p = 0;
        phase_setup();
    }
    finish_pending();
    flush_stats();
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
    if ((((uintptr_t)x) & 15u) || (((uintptr_t)z) & 15u) || (((uintptr_t)ws) & 15u) || (((uintptr_t)w) & 15u)) return LAMP_ERR_ALIGN;
    const int td = (zd->d + RTD - 1) / RTD, th = (zd->h + RTH - 1) / RTH, tw = (zd->w + RTW - 1) / RTW;
    const int tiles_per_n = td * th * tw;
    Carver cv(ws, ws_bytes);
    bf16_t* wp = (bf16_t*)cv.take((size_t)27 * xd->c * zd->c * 2 + 2 * xd->c + 64);
    // launch shape first: the statistics partials are per wave of a workgroup ([N][4 * workgroups][C][2])
    const int tiles_total = tiles_per_n * zd->n;
    const int tiles_per_xcd = (tiles_total + 7) / 8;
    int wg_per_xcd = tiles_per_xcd < 32 ? tiles_per_xcd : 32;  // one persistent workgroup per CU (LDS-limited)
    const int tiles_per_wg = (tiles_per_xcd + wg_per_xcd - 1) / wg_per_xcd;
    wg_per_xcd = (tiles_per_xcd + tiles_per_wg - 1) / tiles_per_wg;
    const int sparts = 8 * wg_per_xcd * 4;
    float* part = nullptr;
    int32_t* counts = nullptr;
    if (stats_out) {
        part = (float*)cv.take((size_t)zd->n * sparts * zd->c * 2 * sizeof(float));
        counts = (int32_t*)cv.take((size_t)zd->n * sparts * sizeof(int32_t));
    }
    if (!cv.ok()) return LAMP_ERR_WORKSPACE;
    const int cob = (zd->c % 64 == 0) ? 2 : 1;
    const int64_t wtotal = (int64_t)27 * xd->c * zd->c;
    if (const bf16_t* pre = find_prepacked(w, dgrad, cob == 2 ? 2 : 3, zd->c, xd->c)) {
        wp = const_cast<bf16_t*>(pre);
    } else {
        hipLaunchKernelGGL(ring_repack_kernel, dim3(cdiv(wtotal / 8, 256)), dim3(256), 0, s, (const bf16_t*)w, wp, zd->c, xd->c,
                           32 * cob, dgrad ? 1 : 0);
        LAMP_CHECK_LAUNCH();
    }
    RingArgs a;
    a.x = (const bf16_t*)x; a.ldx = xd->ldc; a.wp = wp; a.z = (bf16_t*)z; a.ldz = zd->ldc; a.part = part; a.counts = counts;
    a.zero16 = wp + (size_t)27 * xd->c * zd->c;
    a.dump = wp + (size_t)27 * xd->c * zd->c + xd->c + 16;
    a.N = zd->n; a.D = zd->d; a.H = zd->h; a.W = zd->w; a.Cin = xd->c; a.Cout = zd->c;
    a.tiles_d = td; a.tiles_h = th; a.tiles_w = tw; a.tiles_per_n = tiles_per_n;
    a.tiles_total = tiles_total; a.tiles_per_xcd = tiles_per_xcd; a.tiles_per_wg = tiles_per_wg;
    dim3 grid(8 * wg_per_xcd, zd->c / (32 * cob));
    lamp_status st = cob == 2 ? launch_ring<2>(a, grid, s) : launch_ring<1>(a, grid, s);
    if (st != LAMP_OK) return st;
    if (stats_out) return launch_stats_finalize(part, counts, sparts, zd->n, zd->c, eps, stats_out, s, true);
    return LAMP_OK;
}

}  // namespace lamp
