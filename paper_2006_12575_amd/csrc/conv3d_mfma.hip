// Matrix-core (MFMA) implicit-GEMM 3x3x3 convolution kernels for gfx950, bf16 in / fp32 accumulate.
//
// Forward and data-gradient share one kernel (the data gradient is a forward convolution with
// spatially flipped taps and swapped channel roles, done by the weight repack).
//
// GEMM view per workgroup tile:  D[co][voxel] += sum_{tap, ci} Wp[tap][co][ci] * X[voxel + tap][ci]
//   M = 32*COB output channels (A operand = weights), N = 1024 voxels (B operand = activations),
//   K = 27 taps x Cin, walked as (Cin chunk of 16 = one MFMA k-step) x (3 groups of 9 taps, one in-plane row kh
//   each) x (3 tap columns kw of 3 taps kd).
// Tile: 8 x 8 x 16 (or 4 x 8 x 16) output voxels (d,h,w); 8 waves (2 per SIMD); a wave owns 4 (2) d-slices of one
// (2 h-rows x 16 w) patch = 4 (2) blocks of 32 voxels, so a 16-lane group always reads 16 consecutive
// halo voxels and an input slice fragment serves up to three output slices (kd = 0, 1, 2).
// LDS holds a halo chunk as 32-byte voxel entries (the two 16-byte halves = channels 0-7 / 8-15 of the chunk, in
// swapped order where bit 3 of the halo w coordinate is set): a copy instruction fetches both halves of 32 voxels,
// so two lanes share every line they touch, and every fragment read is a conflict-free 16-byte load at a lane base
// (one per tap column kw) plus an immediate offset.
// Two halo buffers (10 x 10 x 18 voxels) let the next chunk / next tile stream in while the
// current one is multiplied; two weight buffers hold one tap group (9 taps x 64 or 32 co x 16 ci) each.
// Workgroups are persistent and walk an XCD-contiguous range of tiles.
#include <stdlib.h>
#include "internal.h"
#include <type_traits>
#include "repack.h"

namespace lamp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

static constexpr int TH = 8, TW = 16;
static constexpr int HH = TH + 2, HW = TW + 2;

// Tile geometry for a tile depth of TDT (8 or 4) output d-slices.  The 8 waves split the tile as 2 halves in d x 4
// pairs of h-rows (h, h + 4); a wave owns TDT/2 consecutive d-slices of its row pair, one block of 32 voxels
// (2 h-rows x 16 w) each.
template <int TDT> struct Geo {
    static constexpr int TD = TDT, HD = TDT + 2;
    static constexpr int ND = TDT / 2, NVB = ND;             // d-slices (= blocks of 32 voxels) per wave: 4 / 2
    static constexpr int HALO_VOX = HD * HH * HW;            // 1800 / 1080
    static constexpr int HALO_BYTES = HALO_VOX * 32;         // one 16-channel chunk, 32 bytes per voxel entry
    static constexpr int HBLK = (HALO_VOX + 31) / 32;        // wave-wide copies per halo chunk (32 voxels each): 57 / 34
    static constexpr int HJ = (HBLK + 7) / 8;                // copy slots per wave (slot j = block wv + 8*j): 8 / 5
    static constexpr int ALLW = (HALO_VOX / 32) / 8;         // slots that every wave issues, in full: 7 / 4
};

// LDS layout of a workgroup: two halo buffers (one 16-channel chunk each), two weight buffers (one in-plane row of 9
// taps x 16 input channels x the output-channel block), the epilogue's patches, the channel sums, the coefficient table.
template <int TDT, int COB> struct Lds {
    typedef Geo<TDT> GE;
    static constexpr int WBUF_BYTES = 9 * 2 * (32 * COB) * 16;      // 9216 / 18432
    static constexpr int W_OFF = 2 * GE::HALO_BYTES;
    // Epilogue scratch: per wave a patch of 32 voxel rows (the output-channel block plus 16 bytes of padding each).
    // With a 32-channel block the epilogue of a tile runs during the multiply of the next one, when both halo buffers
    // are in use: its patches have a region of their own.  With 64 channels the patches take the halo buffer of the
    // stage just finished, where that is large enough (the 8-deep tile).
    static constexpr int ROWB = 32 * COB * 2 + 16;
    static constexpr int PATCH_BYTES = 8 * 32 * ROWB;               // 20480 / 36864
    static constexpr bool EPI_OWN = COB == 1 || GE::HALO_BYTES < PATCH_BYTES;
    static constexpr int PATCH_OFF = W_OFF + 2 * WBUF_BYTES;
    // the channel sums of each wave (64 channels x (sum, sum of squares)) outlive the epilogue: they are added up
    // behind a later barrier
    static constexpr int SUMS_OFF = PATCH_OFF + (EPI_OWN ? PATCH_BYTES : 0), SUMS_BYTES = 8 * 64 * 2 * 4;
    // normalise on load: the (a, b) pairs of the incoming chunk's 16 channels
    static constexpr int TAB_OFF = SUMS_OFF + SUMS_BYTES, TAB_BYTES = 128;
    static constexpr int LDS_BYTES = TAB_OFF + TAB_BYTES;
    static_assert(LDS_BYTES <= 160 * 1024, "the layout fits the LDS of a compute unit");
};

// Two floats to a pair of bf16 (round to nearest even) with the hardware conversion.
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
// v of the lane N places further round in its row of 16 lanes (a DPP row rotation).
template <int N> __device__ __forceinline__ float row_ror(float v) {
    const int r = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x120 + N, 0xF, 0xF, false);
    return __builtin_bit_cast(float, r);
}
__device__ __forceinline__ bf16x8 lds_frag(const char* p) {
    uint4 q = *reinterpret_cast<const uint4*>(p);
    return __builtin_bit_cast(bf16x8, q);
}

__global__ __launch_bounds__(256) void repack_weights_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wp,
                                                             int Cout, int Cin, int dgrad, int bykh) {
    repack_tile_gran(w, wp, (int64_t)blockIdx.x * 256 + threadIdx.x, Cout, Cin, Cout % 64 == 0 ? 64 : 32, dgrad, bykh);
}

// All the repacks of a network pass in one launch: block -> job by the jobs' first-block table.
struct RepackBatch {
    int n;
    struct J { const bf16_t* w; bf16_t* wp; int Cout, Cin, dgrad, kind, blk0; } j[64];
};
__global__ __launch_bounds__(256) void repack_batch_kernel(RepackBatch b) {
    int k = 0;
    while (k + 1 < b.n && (int)blockIdx.x >= b.j[k + 1].blk0) ++k;
    const RepackBatch::J& q = b.j[k];
    const int64_t i = (int64_t)((int)blockIdx.x - q.blk0) * 256 + threadIdx.x;
    repack_tile_gran(q.w, q.wp, i, q.Cout, q.Cin, q.Cout % 64 == 0 ? 64 : 32, q.dgrad, q.kind);
}

lamp_status launch_repack_batch(const RepackJob* jobs, int n, hipStream_t s) {
    if (n <= 0) return LAMP_OK;
    if (n > 64) return LAMP_ERR_SHAPE;
    RepackBatch b;
    b.n = n;
    int64_t blk = 0;
    for (int k = 0; k < n; ++k) {
        b.j[k].w = (const bf16_t*)jobs[k].w; b.j[k].wp = (bf16_t*)jobs[k].wp;
        b.j[k].Cout = jobs[k].Cout; b.j[k].Cin = jobs[k].Cin; b.j[k].dgrad = jobs[k].dgrad; b.j[k].kind = jobs[k].kind;
        b.j[k].blk0 = (int)blk;
        blk += cdiv((int64_t)27 * jobs[k].Cout * jobs[k].Cin / 8, 256);
        if (blk >= ((int64_t)1 << 31)) return LAMP_ERR_SHAPE;
    }
    hipLaunchKernelGGL(repack_batch_kernel, dim3((unsigned)blk), dim3(256), 0, s, b);
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}

static thread_local const RepackTable* tl_repack = nullptr;
void set_repack_table(const RepackTable* t) { tl_repack = t; }
const bf16_t* find_prepacked(const void* w, bool dgrad, int kind, int Cout, int Cin) {
    const RepackTable* t = tl_repack;
    if (!t) return nullptr;
    for (int k = 0; k < t->n; ++k)
        if (t->e[k].w == w && (t->e[k].dgrad != 0) == dgrad && t->e[k].kind == kind && t->e[k].Cout == Cout && t->e[k].Cin == Cin) return (const bf16_t*)t->e[k].wp;
    return nullptr;
}

struct ConvArgs {
    const bf16_t* x; int ldx;
    const bf16_t* wp;
    bf16_t* z; int ldz;
    float* part;        // [N][tiles_per_n][Cout][2] or nullptr
    int32_t* counts;    // [tiles_per_n] in-volume voxels per tile (written when part != nullptr)
    // 32-channel block with long walks: one partial per (sample, workgroup walk) instead of per tile -- part is
    // [N][walk_parts][Cout][2], counts [N][walk_parts] (0 where a walk holds no tile of the sample); 0: per tile
    int walk_parts;
    const bf16_t* zero16;  // 16 zero bytes in global memory (source of the zero padding)
    const float* bias;     // [Cout] fp32 added to the accumulators before rounding and the statistics, or nullptr
    // Normalise + ReLU while loading (NORM instantiations): per (sample, input channel) the pair (a, b) of
    // u = a*x + b, a = gamma*rstd, b = beta - mean*a; relu_floor = 0 (ReLU) or -inf (none).
    const float2* ab;
    float relu_floor;
    // Data gradient with the two sums of the InstanceNorm + ReLU backward of the layer below (BSUM instantiations):
    // zb = that layer's raw conv output z, whose activation u = a*z + b (zab: the (a, b) pairs per (sample, channel))
    // fed this conv in the forward -- the voxels, channels and channel stride of the tensor written here.  With
    // g = [u > 0] * dx (dx = the value stored, after rounding) the per-tile partials hold (sum g, sum g*z).
    const bf16_t* zb;
    const float2* zab;
    int N, D, H, W, Cin, Cout;
    int tiles_d, tiles_h, tiles_w, tiles_per_n, tiles_total, tiles_per_xcd;
    float* zpart;       // split reduction only: [splits][N*D*H*W][Cout] fp32 partial outputs
    int cps;            // split reduction only: 16-channel input chunks per split (grid z = split)
    // Two-part tensors (a concat that is never materialised).  Input: the 16-channel chunks from xsplit on
    // are read from x + xdelta (an element offset to the second tensor, same channel stride).  Output:
    // channels from zsplit on go to z2 (channel stride ldz2), counted from its channel 0.
    int64_t xdelta; int xsplit;
    bf16_t* z2; int ldz2, zsplit;
    // With very few tiles only the first XCD ranges hold work, and a workgroup's XCD is its flattened id
    // modulo 8 = blockIdx.x & 7: rotating the range a workgroup serves by its channel-block / split index
    // spreads the channel blocks of those few tiles over all eight XCDs.
    int xcd_rot;
    // Output-channel blocks inside a one-dimensional grid: workgroup id = (walker * cb_inner + channel block) * 8 + XCD,
    // so the workgroups that read the same tiles for different output channels are resident on the same XCD at
    // the same time and share the input through its L2.  0: the channel block is blockIdx.y (they run one after
    // the other when the grid exceeds the chip).
    int cb_inner;
};

// 16-byte global -> LDS copy that bypasses registers: lane l's 16 bytes land at lds_base + 16*l
// (lds_base must be wave-uniform); inactive lanes write nothing.  Issued as inline assembly so that
// the compiler's wait-count bookkeeping does not see it: with the builtin form every later wait for an
// LDS fragment read degrades to "wait for all reads".  Completion is tracked by hand with wait_vmcnt.
__device__ __forceinline__ void g2lds16(const void* g, char* lds_base) {
    const uint32_t m = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds_base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(m), "v"(g) : "memory", "m0");
}

// The same with the target given as an LDS byte address (kept as an integer from the start, so that no pointer
// passes through the generic address space on its way here).
__device__ __forceinline__ void g2lds16a(const void* g, uint32_t lds_addr) {
    const uint32_t m = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(m), "v"(g) : "memory", "m0");
}

// Scheduling hint: NM MFMAs with NR LDS reads spread evenly behind them.
template <int K, int NM, int NR> __device__ __forceinline__ void sched_interleave() {
    if constexpr (K < NM) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        constexpr int R = (NR * (K + 1)) / NM - (NR * K) / NM;
        if constexpr (R > 0) __builtin_amdgcn_sched_group_barrier(0x100, R, 0);
        sched_interleave<K + 1, NM, NR>();
    }
}

template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }


// Per-lane constants of the halo copies.  A wave copies halo blocks wv, wv + 8, ... (32 voxels each; lanes 2i and
// 2i + 1 fetch the two 16-byte halves of voxel i's 32 bytes, in the order the LDS entry stores them).  pk = the halo
// coords of the lane's voxel, 16 bits a slot, two slots to a register (slot j in the low or high half of pk[j / 2]):
// d in bits 0-3, h in bits 5-8, w in bits 10-14, and a guard bit above each field (bits 4, 9, 15), so that one
// subtraction compares all three coordinates of both slots with a bound: a field's guard bit survives
// (c + guard) - lo exactly when c >= lo, and (hi + guard) - c exactly when c <= hi, and never borrows from its
// neighbour.  Six compares and five mask operations per slot become four instructions.
static constexpr uint32_t HALO_GUARD = 0x8210u, HALO_GUARD2 = 0x82108210u;
struct HaloTile {
    const bf16_t* origin;   // x at the halo origin (d0-1, h0-1, w0-1) of the tile (may be out of range)
    uint32_t lo2, hi2;      // halo coords inside the volume, lo <= c <= hi per field, packed like HaloLane::pk (no guards)
};
struct HaloLane {
    int pk[4];
    int rel[8];   // element offset of the lane's 16 bytes from the tile's halo origin (kernels with registers to spare)
    // which half (plane) of the chunk's channels the lane fetches for slot j follows from its voxel's w
    template <bool LEAN> __device__ __forceinline__ void coords(int j, int lane, int& hd, int& hh, int& hw, int& plane) const {
        int v = (j & 1) ? pk[j >> 1] >> 16 : pk[j >> 1];
        // LEAN (the 64-channel kernel of the 8-deep tile, which has no register to spare): opaque, because what is
        // derived from the coordinates (the voxel's offset in the tensor) is cheap to recompute at every use, where
        // the compiler would rather compute all of it once and keep it in registers it has not got
        if constexpr (LEAN) asm volatile("" : "+v"(v));
        hd = v & 15; hh = (v >> 5) & 15; hw = (v >> 10) & 31; plane = (lane & 1) ^ ((hw >> 3) & 1);
    }
    // whether the voxel of slot j lies inside the volume
    __device__ __forceinline__ bool inside(int j, const HaloTile& ht) const {
        const uint32_t p = (uint32_t)pk[j >> 1];
        const uint32_t t = (p - ht.lo2) & ((ht.hi2 | HALO_GUARD2) - (p ^ HALO_GUARD2));
        const uint32_t g = (j & 1) ? HALO_GUARD << 16 : HALO_GUARD;
        return (t & g) == g;
    }
};

// Normalise + ReLU on load: the halo copies are register-free, so the transform is a read-modify-write pass over
// the chunk once it has landed in LDS.  Every lane rewrites the 16-byte pieces (8 channels of one voxel) that
// its own copies brought in -- it knows whether each came from the volume or from the zero source, and the zero
// padding applies AFTER the transform, so padding entries are written back as literal zeros.  The arithmetic is
// the one of the stand-alone pass (fma, max, round to nearest even), so what the matrix cores read is bit for
// bit the activated tensor that pass would have stored.  tab: the (a, b) pairs of this chunk's 16 channels in LDS
// (a lane's half of the channels depends on its voxel).
template <int TDT, int FIRST, int CNT>
__device__ __forceinline__ void halo_norm(char* __restrict__ hb, const HaloLane& hl, const HaloTile& ht,
                                          const char* __restrict__ tab, float relu_floor, int wv, int lane) {
    typedef Geo<TDT> GE;
#pragma unroll
    for (int j = FIRST; j < FIRST + CNT; ++j) {
        const int blk = wv + 8 * j;
        int hd, hh, hw, plane;
        hl.template coords<true>(j, lane, hd, hh, hw, plane);
        const bool in = hl.inside(j, ht);
        // Slots that every wave copies in full are rewritten by straight-line code; an entry from outside the volume
        // is written back as it came (zeros: the zero padding applies after the transform).  The last slots exist
        // for some waves and lanes only.
        const bool mine = j < GE::ALLW || (blk < GE::HBLK && blk * 32 + (lane >> 1) < GE::HALO_VOX);
        if (mine) {
            uint4* p = reinterpret_cast<uint4*>(hb + blk * 1024 + lane * 16);
            const uint4 q = *p;
            const uint32_t r[4] = {q.x, q.y, q.z, q.w};
            uint32_t o[4];
            const float4* cab = reinterpret_cast<const float4*>(tab + plane * 64);   // (a, b) pairs of the lane's 8 channels
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float4 c = cab[e];
                // max(u, floor): for u = -0 the sign of the zero may differ from the stand-alone pass, which
                // the matrix cores cannot see (both are zero)
                const float u0 = fmaxf(fmaf(__uint_as_float(r[e] << 16), c.x, c.y), relu_floor);
                const float u1 = fmaxf(fmaf(__uint_as_float(r[e] & 0xFFFF0000u), c.z, c.w), relu_floor);
                o[e] = in ? pack_bf16(u0, u1) : r[e];
            }
            *p = make_uint4(o[0], o[1], o[2], o[3]);
        }
    }
}

// Scheduling hint: NM MFMAs with NR LDS reads, NV vector-ALU instructions and NW LDS writes spread evenly behind them.
template <int K, int NM, int NR, int NV, int NW> __device__ __forceinline__ void sched_interleave_v() {
    if constexpr (K < NM) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        constexpr int R = (NR * (K + 1)) / NM - (NR * K) / NM;
        if constexpr (R > 0) __builtin_amdgcn_sched_group_barrier(0x100, R, 0);
        constexpr int V = (NV * (K + 1)) / NM - (NV * K) / NM;
        if constexpr (V > 0) __builtin_amdgcn_sched_group_barrier(0x002, V, 0);
        constexpr int Wr = (NW * (K + 1)) / NM - (NW * K) / NM;
        if constexpr (Wr > 0) __builtin_amdgcn_sched_group_barrier(0x200, Wr, 0);
        sched_interleave_v<K + 1, NM, NR, NV, NW>();
    }
}

// Fragment registers that live from one column of the multiply pipeline to the next (and from the last column of
// a tile, across its epilogue, to the first column of the next tile).
template <int COB> struct Frags {
    bf16x8 a[2][3][COB];   // weight fragments of a tap column (kd = 0, 1, 2), two slots
    bf16x8 b[2];           // input slices 0 and 1 of the current column
};

// The fragments of the first column of group G, into slot SLOT.
template <int COB, int G, int SLOT>
__device__ __forceinline__ void load_first(Frags<COB>& f, const char* __restrict__ hbu, const char* __restrict__ wb,
                                           const uint32_t (&boff)[3]) {
    constexpr int WPLANE = 32 * COB * 16;
    const char* hb = hbu + boff[0];
#pragma unroll
    for (int kd = 0; kd < 3; ++kd)
#pragma unroll
        for (int cb = 0; cb < COB; ++cb) f.a[SLOT][kd][cb] = lds_frag(wb + (kd * 3) * 2 * WPLANE + cb * 32 * 16);
    f.b[0] = lds_frag(hb + ((0 * HH + G) * HW) * 32);
    f.b[1] = lds_frag(hb + ((1 * HH + G) * HW) * 32);
}

// What the register-free copies and the normalise-on-load rewrite of a chunk stage need.
struct CopyCtx {
    char* hb_next;          // halo buffer of the incoming chunk
    uint32_t hb_next_a;     // its LDS byte address
    uint32_t wb_fill_a;     // LDS byte address of the weight buffer that this group has finished with
    bool pf_halo, pf_w;     // whether there is an incoming chunk / a weight group to fetch
    int64_t pf_choff;       // element offset of the incoming chunk's channels
    const bf16_t* zero16;
    const bf16_t* wsrc;     // weights of the group after next
    const float2* abp;      // normalise on load: (a, b) pairs of the incoming chunk's channels (global memory)
    const char* tab;        // ... and where they go in LDS
    uint32_t tab_a;
    float relu_floor;
    int H, W, ldx;          // strides of the input tensor
    int wv, lane;
};

// One halo copy slot: 32 voxels, both halves of their 32 bytes (lanes 2i, 2i + 1 = voxel i).
template <int TDT, bool LEAN>
__device__ __forceinline__ void halo_copy_slot(int j, const HaloLane& hl, const HaloTile& ht, int H, int W, int ldx, int64_t choff,
                                               const bf16_t* zero16, uint32_t hb_a, int wv, int lane) {
    typedef Geo<TDT> GE;
    const int blk = wv + 8 * j;
    if (blk < GE::HBLK && blk * 32 + (lane >> 1) < GE::HALO_VOX) {
        int hd, hh, hw, plane;
        hl.template coords<LEAN>(j, lane, hd, hh, hw, plane);
        const bool in = hl.inside(j, ht);
        // ((hd*H + hh)*W + hw)*ldx with 24-bit multiply-adds (full rate, where a 32-bit multiply takes four passes):
        // hd*H + hh and W*ldx stay below 2^24 (checked on the host)
        const int rel = LEAN ? (int)(__umul24(__umul24(hd, H) + hh, W * ldx) + __umul24(hw, ldx) + plane * 8) : hl.rel[j];
        const bf16_t* src = in ? ht.origin + rel + choff : zero16;
        g2lds16a(src, hb_a + blk * 1024);
    }
}

// One portion of a stage's copy work, placed in the middle of a column's matrix instructions (the global -> LDS
// copies of a wave queue up behind each other: issued in one burst they hold up the wave, and with it the
// workgroup's next barrier, for thousands of cycles; a few per column never fill the queue):
//   WC          : the weight copies of the group after next
//   HF, HC      : halo copy slots [HF, HF + HC) of the incoming chunk (slot j = block wv + 8*j of 32 voxels)
//   NF, NC, NW  : normalise on load: rewrite slots [NF, NF + NC) once at most NW of this wave's copies are in flight
template <int COB, int TDT, bool WC, int HF, int HC, int NF, int NC, int NW, bool TABC>
__device__ __forceinline__ void copy_portion(const CopyCtx& c, const HaloLane& hl, const HaloTile& ht, const int (&wrel)[3]) {
    typedef Geo<TDT> GE;
    constexpr int WINSTR = 18 * 32 * COB / 64;
    constexpr int WCOPY_ITERS = (WINSTR + 7) / 8;
    if constexpr (NC > 0) {
        if (c.pf_halo) {
            wait_vmcnt<NW>();
            halo_norm<TDT, NF, NC>(c.hb_next, hl, ht, c.tab, c.relu_floor, c.wv, c.lane);
        }
    }
    if constexpr (TABC) {
        // normalise on load: the incoming chunk's 16 (a, b) pairs, 128 bytes, older than every copy whose landing is
        // counted (wave 0, lanes 0..7)
        if (c.pf_halo && c.wv == 0 && c.lane < 8) g2lds16a(reinterpret_cast<const char*>(c.abp) + c.lane * 16, c.tab_a);
    }
    if constexpr (WC) {
        if (c.pf_w) {
#pragma unroll
            for (int i = 0; i < WCOPY_ITERS; ++i) {
                const int q = c.wv + 8 * i;
                if (q < WINSTR) g2lds16a(c.wsrc + wrel[i], c.wb_fill_a + q * 1024);
            }
        }
    }
    if constexpr (HC > 0) {
        if (c.pf_halo) {
#pragma unroll
            for (int j = HF; j < HF + HC; ++j)
                halo_copy_slot<TDT, (COB == 2 && TDT == 8)>(j, hl, ht, c.H, c.W, c.ldx, c.pf_choff, c.zero16, c.hb_next_a, c.wv, c.lane);
        }
    }
}

// Which portion goes where.  The halo of the incoming chunk may be written once every wave is past the barrier of the
// chunk's group 0 (the previous chunk's halo, whose buffer it takes, is read up to the column before), and must have
// landed at the barrier of group 2, so its slots go out between the last column of group 0 and the last column of
// group 1, leaving the youngest ones three columns to land.  The column in front of a barrier carries nothing: the
// wave that reaches the barrier last would do that work with the matrix cores idle.
// COL: tap column of the group.
struct PortionSpec { bool wc; int hf, hc, nf, nc, nw; bool tab; };
template <int TDT, bool NORM> constexpr PortionSpec portion_spec(int G, int COL) {
    constexpr int NS = Geo<TDT>::HJ, ALLW = Geo<TDT>::ALLW;   // 8 / 5 slots, of which every wave issues the first 7 / 4
    const int last = 2;                             // the column behind the barrier
    PortionSpec p{COL == last, 0, 0, 0, 0, 0, false};
    if (!NORM) {
        if (G == 0 && COL == 2) { p.hf = 0; p.hc = 2; }
        if (TDT == 8) {
            if (G == 1 && COL == 0) { p.hf = 2; p.hc = 4; }
            if (G == 1 && COL == 2) { p.hf = 6; p.hc = 2; }
        } else {
            if (G == 1 && COL == 0) { p.hf = 2; p.hc = 3; }
        }
    } else {
        // Normalise on load: the copies go out earlier, and the entries they brought in are rewritten three columns
        // later.  First rewrite: younger than slot 3 are the all-wave slots from 4 on; second one: the weight copies
        // that went out with the first, of which every wave issues at least one.  The coefficient table goes out with
        // the first slots, ahead of the weight copies.
        if (G == 0 && COL == last) { p.hf = 0; p.hc = 4; p.tab = true; }
        if (G == 1 && COL == 0) { p.hf = 4; p.hc = NS - 4; }
        if (G == 1 && COL == last) { p.nf = 0; p.nc = 4; p.nw = ALLW - 4; }
        if (G == 2 && COL == 0) { p.nf = 4; p.nc = NS - 4; p.nw = 1; }
    }
    return p;
}
// Copies of a wave that may be in flight at a group's barrier without the next group's weights among them: at the
// barrier of group 1, the all-wave halo slots issued behind the weight copies of (group 0, last column).
template <int TDT, bool NORM> constexpr int barrier_wait(int G) {
    return G != 1 ? 0 : NORM ? Geo<TDT>::ALLW : TDT == 8 ? 6 : 4;
}

// One tap column kw = KW of the in-plane row G = kh.  A wave owns ND = 4 (8-deep tile) or 2 (4-deep tile) d-slices of
// one (2 h-rows x 16 w) block; the input slice s = d + kd serves the output slices d = s, s-1, s-2 with the weights of
// kd = 0, 1, 2: ND + 2 slice fragments and 3*COB weight fragments feed 3*ND*COB MFMAs.  The weight fragments and the
// first two slices of the next column are fetched meanwhile: of column KW + 1, or (KW == 2) of the first column of the
// group GN that follows, whose weights sit in wbn and whose halo is hbn.  The column's portion of the copy work
// follows its matrix instructions.
// ZERO: the first column of a tile -- every accumulator's first matrix instruction (its tap kd = 0) takes zero as its
// addend, so nothing has to clear the accumulators between tiles.
template <int COB, int TDT, int G, int KW, int SLOT, int GN, bool NORM, bool ZERO = false>
__device__ __forceinline__ void column(f32x16 (&acc)[COB][Geo<TDT>::ND], Frags<COB>& f, const char* __restrict__ hbu,
                                       const char* __restrict__ wb, const char* __restrict__ hbnu, const char* __restrict__ wbn,
                                       const uint32_t (&boff)[3], const CopyCtx& c, const HaloLane& hl, const HaloTile& ht,
                                       const int (&wrel)[3]) {
    constexpr int WPLANE = 32 * COB * 16, ND = Geo<TDT>::ND;
    // lane bases of this tap column and of the one fetched ahead (the half of a voxel's entry that holds the lane's
    // channels depends on the voxel's w coordinate, and with it on kw)
    const char* hb = hbu + boff[KW];
    const char* hbx = KW < 2 ? hbu + boff[KW + 1] : hbnu + boff[0];
    constexpr PortionSpec PO = portion_spec<TDT, NORM>(G, KW);
    bf16x8 b[ND + 2], nb0, nb1;
    b[0] = f.b[0];
    b[1] = f.b[1];
#pragma unroll
    for (int sl = 2; sl < ND + 2; ++sl) b[sl] = lds_frag(hb + ((sl * HH + G) * HW) * 32);
    if constexpr (KW < 2) {
#pragma unroll
        for (int kd = 0; kd < 3; ++kd)
#pragma unroll
            for (int cb = 0; cb < COB; ++cb) f.a[SLOT ^ 1][kd][cb] = lds_frag(wb + (kd * 3 + KW + 1) * 2 * WPLANE + cb * 32 * 16);
        nb0 = lds_frag(hbx + ((0 * HH + G) * HW) * 32);
        nb1 = lds_frag(hbx + ((1 * HH + G) * HW) * 32);
    } else {
#pragma unroll
        for (int kd = 0; kd < 3; ++kd)
#pragma unroll
            for (int cb = 0; cb < COB; ++cb) f.a[SLOT ^ 1][kd][cb] = lds_frag(wbn + (kd * 3) * 2 * WPLANE + cb * 32 * 16);
        nb0 = lds_frag(hbx + ((0 * HH + GN) * HW) * 32);
        nb1 = lds_frag(hbx + ((1 * HH + GN) * HW) * 32);
    }
#pragma unroll
    for (int sl = 0; sl < ND + 2; ++sl)
#pragma unroll
        for (int kd = 0; kd < 3; ++kd) {
            const int d = sl - kd;
            if (d >= 0 && d < ND) {
#pragma unroll
                for (int cb = 0; cb < COB; ++cb) {
                    if constexpr (ZERO) {
                        if (kd == 0) {
                            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                            acc[cb][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[SLOT][kd][cb], b[sl], zero, 0, 0, 0);
                            continue;
                        }
                    }
                    acc[cb][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[SLOT][kd][cb], b[sl], acc[cb][d], 0, 0, 0);
                }
            }
        }
    sched_interleave<0, 3 * ND * COB, ND + 2 + 3 * COB>();
    if constexpr (PO.wc || PO.hc > 0 || PO.nc > 0) {
        // behind the column's last matrix instruction, where the fewest fragments are live
        __builtin_amdgcn_sched_barrier(0);
        copy_portion<COB, TDT, PO.wc, PO.hf, PO.hc, PO.nf, PO.nc, PO.nw, PO.tab>(c, hl, ht, wrel);
        __builtin_amdgcn_sched_barrier(0);
    }
    f.b[0] = nb0;
    f.b[1] = nb1;
}

// One tap group of one chunk (9 taps: the in-plane row kh = G, three tap columns kw).  The multiply runs as one
// pipeline of columns across groups, chunks and tiles: every column fetches
// the fragments of the next one, so the matrix instructions that follow a barrier have their operands in registers.
// The workgroup's barrier therefore sits BEFORE the group's last column: by then every wave has read the
// last fragments of this group's weights, and all of the previous chunk's halo.  What is copied in behind the
// barrier: the weights of the group after next, into the buffer this group has just finished with (the last column
// fetches the first fragments of the next group from the other weight buffer, filled one group earlier), and
// the next chunk's halo, into the buffer the previous chunk has left (see portion_spec).
//   PAR        : fragment slot of the group's first column (it alternates from column to column)
//   hb, hbn    : halo buffers of this group and of the group that follows (boff: lane bases per tap column kw)
//   wb, wbn    : their weights (lane base included)
// The LDS regions are distinct, and saying so (__restrict__) matters: otherwise the compiler must assume the
// fragment reads alias the in-flight copies and waits for them before the first read.
template <int COB, int TDT, int G, int PAR, bool NORM>
__device__ __forceinline__ void conv_group(f32x16 (&acc)[COB][Geo<TDT>::ND], Frags<COB>& f, const char* __restrict__ hb,
                                           const char* __restrict__ wb, const char* __restrict__ hbn,
                                           const char* __restrict__ wbn, const uint32_t (&boff)[3], const CopyCtx& c,
                                           const HaloLane& hl, const HaloTile& ht, const int (&wrel)[3], bool first = false) {
    constexpr int GN = (G + 1) % 3;
    constexpr int WAIT = barrier_wait<TDT, NORM>(G);
    if (G == 0 && first) column<COB, TDT, G, 0, PAR, GN, NORM, true>(acc, f, hb, wb, hbn, wbn, boff, c, hl, ht, wrel);
    else column<COB, TDT, G, 0, PAR, GN, NORM>(acc, f, hb, wb, hbn, wbn, boff, c, hl, ht, wrel);
    column<COB, TDT, G, 1, PAR ^ 1, GN, NORM>(acc, f, hb, wb, hbn, wbn, boff, c, hl, ht, wrel);
    // The weights of the next group were copied behind the previous barrier; the only younger copies are halo slots,
    // of which every wave has issued WAIT (a wave that issued more waits for its oldest ones too).
    if (WAIT > 0 && c.pf_halo) wait_vmcnt<WAIT>();
    else wait_vmcnt<0>();
    // bare barrier: __syncthreads() would add a release fence that drains every copy in flight
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0), as a builtin so the compiler knows the reads are done
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    column<COB, TDT, G, 2, PAR, GN, NORM>(acc, f, hb, wb, hbn, wbn, boff, c, hl, ht, wrel);
}

// SPLIT: the input-channel chunks are divided among gridDim.z workgroups per tile, each of which
// writes its fp32 partial sums; a second kernel adds them in a fixed order.  For small volumes with
// many channels, where the tiles alone cannot fill the chip.
template <int COB, int TDT, bool SPLIT = false, bool NORM = false, bool BSUM = false>
__global__ __launch_bounds__(512) void conv3d_igemm_kernel(ConvArgs a) {
    typedef Geo<TDT> GE;
    typedef Lds<TDT, COB> LD;
    constexpr bool ZERO_START = COB == 1 && !BSUM;
    constexpr int WBUF_BYTES = LD::WBUF_BYTES;
    constexpr int TD = GE::TD, NVB = GE::NVB, HALO_VOX = GE::HALO_VOX, HALO_BYTES = GE::HALO_BYTES, HJ = GE::HJ;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char* hbuf0 = lds;
    char* wbuf0 = lds + LD::W_OFF;
    // LDS byte addresses of the two, for the register-free copies
    const uint32_t lds_a = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds, wbuf_a = lds_a + LD::W_OFF;
    const uint32_t tab_a = lds_a + LD::TAB_OFF;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int cbi = a.cb_inner ? (int)(blockIdx.x >> 3) % a.cb_inner : (int)blockIdx.y;   // output-channel block
    const int co0 = cbi * (32 * COB);
    const int nchunks = a.Cin >> 4;
    const int c_lo = SPLIT ? (int)blockIdx.z * a.cps : 0;
    const int c_hi = SPLIT ? min(c_lo + a.cps, nchunks) : nchunks;
    // element offset of a 16-channel chunk from channel 0 of the (first) input tensor
    auto choff = [&](int chunk) -> int64_t {
        return chunk < a.xsplit ? (int64_t)chunk * 16 : a.xdelta + (int64_t)(chunk - a.xsplit) * 16;
    };
    constexpr int WROWS = 32 * COB;
    constexpr int WPLANE = WROWS * 16;            // one (tap, plane): WROWS rows of 16 bytes
    constexpr int WINSTR = 18 * WROWS / 64;       // wave-wide copies per kd group: 18 or 9

    // persistent walk over an XCD-contiguous range of tiles
    const int xcd = (blockIdx.x + (a.xcd_rot ? blockIdx.y + blockIdx.z : 0u)) & 7;
    const int local = a.cb_inner ? (int)(blockIdx.x >> 3) / a.cb_inner : (int)(blockIdx.x >> 3);
    const int wg_per_xcd = a.cb_inner ? (int)(gridDim.x >> 3) / a.cb_inner : (int)(gridDim.x >> 3);
    const int tile_lo = xcd * a.tiles_per_xcd;
    const int tile_hi = min(tile_lo + a.tiles_per_xcd, a.tiles_total);

    // ---- lane -> voxel of a 32-voxel block (2 h-rows x 16 w).  A 16-byte LDS read runs at full rate when the 16
    // lanes served together -- the 8-lane groups {0-7,24-31}, then {8-15,16-23}, and the same in the upper half --
    // hit 16 different 16-byte bank groups (a micro-benchmark of the patterns decides).  Groups of 8 lanes take
    // (row0,w0-7) (row1,w0-7) (row1,w8-15) (row0,w8-15), so the lanes served together read 16 consecutive voxels of
    // one halo row, 32 bytes apart: voxels w and w + 8 would meet in a bank group, which is why the two halves of an
    // entry are stored in swapped order where bit 3 of the halo w coordinate is set.  The two rows of a block are h
    // and h + 4 (4 halo rows of 576 bytes = 0 modulo 256; with adjacent rows the read takes a third longer).
    const int g8 = l32 >> 3;
    const int bw = (l32 & 7) + 8 * (g8 >> 1), bh = (g8 ^ (g8 >> 1)) & 1;
    // this wave's part of the tile: d-slices ND*ds .. ND*ds + ND - 1 (one block each) of the h-row pair (hs, hs + 4)
    constexpr int ND = GE::ND;
    const int ds = wv & 1, hs = wv >> 1;
    // lane base per tap column kw: the entry of voxel (.., bw + kw) and, in it, the half that holds this lane's
    // channels (lanes 0-31: channels 0-7 of the chunk, lanes 32-63: 8-15)
    uint32_t boff[3];
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) {
        const int vox = (ND * ds * HH + hs + 4 * bh) * HW + bw + kw;
        boff[kw] = (uint32_t)(vox * 32 + 16 * (half ^ (((bw + kw) >> 3) & 1)));
    }
    const uint32_t a_base = (uint32_t)(half * WPLANE + l32 * 16);

    // ---- per-lane constants of the register-free global -> LDS copies
    HaloLane hl;
#pragma unroll
    for (int j = 0; j < 4; ++j) hl.pk[j] = 0;
#pragma unroll
    for (int j = 0; j < HJ; ++j) {
        int hv = (wv + 8 * j) * 32 + (lane >> 1);
        if (hv >= HALO_VOX) hv = 0;
        const int hw = hv % HW, hh = (hv / HW) % HH, hd = hv / (HW * HH);
        const int plane = (lane & 1) ^ ((hw >> 3) & 1);
        hl.pk[j >> 1] |= (int)((uint32_t)(hd | (hh << 5) | (hw << 10) | HALO_GUARD) << (16 * (j & 1)));
        hl.rel[j] = ((hd * a.H + hh) * a.W + hw) * a.ldx + plane * 8;
    }
    // weight copy q = wv + 8*i of a group: 64 consecutive (entry,row) pairs, entry = tap9*2 + plane.  The
    // repacked weights are the LDS image itself, [co block][chunk][group][entry][row][8]: every copy reads 1 KB
    // of consecutive memory
    int wrel[3];
#pragma unroll
    for (int i = 0; i < 3; ++i) wrel[i] = ((wv + 8 * i) * 64 + lane) * 8;   // (kept as wrel[0] + i * 4096 by the compiler)
    auto tile_origin = [&](int tile, int& n, int& d0, int& h0, int& w0) {
        n = tile / a.tiles_per_n;
        int r = tile - n * a.tiles_per_n;
        w0 = (r % a.tiles_w) * TW;
        r /= a.tiles_w;
        h0 = (r % a.tiles_h) * TH;
        d0 = (r / a.tiles_h) * TD;
    };
    struct TilePos { int n, d0, h0, w0; };
    auto tile_pos = [&](int tile) {
        TilePos p;
        tile_origin(tile, p.n, p.d0, p.h0, p.w0);
        return p;
    };
    // A workgroup's tiles lie wg_per_xcd apart: from one to the next the position advances by a fixed step, added
    // digit by digit in the mixed radix (tiles_w, tiles_h, tiles_d) -- a dozen scalar instructions where the divisions
    // of tile_origin take a hundred, in one dependent chain.
    int step_n, step_d, step_h, step_w;
    tile_origin(wg_per_xcd, step_n, step_d, step_h, step_w);
    const int lim_d = a.tiles_d * TD, lim_h = a.tiles_h * TH, lim_w = a.tiles_w * TW;
    auto tile_step = [&](const TilePos& p) {
        TilePos q;
        q.w0 = p.w0 + step_w;
        int c = q.w0 >= lim_w ? 1 : 0;
        q.w0 -= c ? lim_w : 0;
        q.h0 = p.h0 + step_h + c * TH;
        c = q.h0 >= lim_h ? 1 : 0;
        q.h0 -= c ? lim_h : 0;
        q.d0 = p.d0 + step_d + c * TD;
        c = q.d0 >= lim_d ? 1 : 0;
        q.d0 -= c ? lim_d : 0;
        q.n = p.n + step_n + c;
        return q;
    };
    auto halo_tile = [&](const TilePos& p) {
        HaloTile t;
        // (a position past the last tile is never read from: its origin only has to be computable)
        const int vox = (((p.n * a.D + (p.d0 - 1)) * a.H + (p.h0 - 1)) * a.W + (p.w0 - 1));
        t.origin = a.x + (int64_t)vox * a.ldx;
        // halo coords c = voxel coordinate - (origin - 1): inside the volume for 1 - origin <= c <= extent - origin
        const uint32_t lo = (uint32_t)(max(1 - p.d0, 0) | (max(1 - p.h0, 0) << 5) | (max(1 - p.w0, 0) << 10));
        const uint32_t hi = (uint32_t)(min(a.D - p.d0, 15) | (min(a.H - p.h0, 15) << 5) | (min(a.W - p.w0, 31) << 10));
        t.lo2 = lo | (lo << 16);
        t.hi2 = hi | (hi << 16);
        return t;
    };
    constexpr int wgstride = 18 * WROWS * 8;                                       // elements of one group
    const bf16_t* wbase = a.wp + (int64_t)cbi * nchunks * (3 * wgstride);    // + (chunk*3 + g) * wgstride

    // Statistics per walk (32-channel block): the channel sums stay in registers from tile to tile, and are folded
    // and written when the walk ends or moves on to the next sample -- not once per tile, where the fold and the
    // write are a twentieth of that kernel's instructions.
    constexpr bool WALK_OK = COB == 1 && !SPLIT && !BSUM;
    const bool walk = WALK_OK && a.walk_parts > 0;
    const int walker = xcd * wg_per_xcd + local;
    int tile = tile_lo + local;
    if (tile >= tile_hi) {
        if (walk && a.counts && tid == 0 && cbi == 0)
            for (int n = 0; n < a.N; ++n) a.counts[n * a.walk_parts + walker] = 0;
        return;
    }
    const int first_n = tile / a.tiles_per_n;
    int last_n = first_n, wcount = 0;
    float ksum[WALK_OK ? 8 : 1], ksq[WALK_OK ? 8 : 1];
#pragma unroll
    for (int e = 0; e < (WALK_OK ? 8 : 1); ++e) { ksum[e] = 0.f; ksq[e] = 0.f; }

    // Where the tile of this pass and the one after it lie.  The position of the tile after those is worked out during
    // the epilogue, whose LDS round trips leave the scalar unit idle: at the top of a pass it would hold up the first
    // matrix instructions of every wave.
    TilePos pos = tile_pos(tile);
    TilePos pos_next = tile_step(pos);
    HaloTile ht_cur = halo_tile(pos), ht_next = halo_tile(pos_next);

    // ---- prologue: first halo chunk and the first two weight groups
    {
        const HaloTile t0 = ht_cur;
#pragma unroll
        for (int j = 0; j < HJ; ++j) halo_copy_slot<TDT, (COB == 2 && TDT == 8)>(j, hl, t0, a.H, a.W, a.ldx, choff(c_lo), a.zero16, lds_a, wv, lane);
        if constexpr (NORM) {
            if (wv == 0 && lane < 8)
                g2lds16a(reinterpret_cast<const char*>(a.ab + (int64_t)pos.n * a.Cin + c_lo * 16) + lane * 16, tab_a);
        }
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int i = 0; i < 3; ++i)
                if (wv + 8 * i < WINSTR)
                    g2lds16a(wbase + (int64_t)c_lo * (3 * wgstride) + g * wgstride + wrel[i], wbuf_a + g * WBUF_BYTES + (wv + 8 * i) * 1024);
        wait_vmcnt<0>();
        if constexpr (NORM) {
            __syncthreads();   // the coefficient table (wave 0's copy) is there for every wave
            halo_norm<TDT, 0, HJ>(hbuf0, hl, t0, lds + LD::TAB_OFF, a.relu_floor, wv, lane);
        }
        __syncthreads();
    }

    int stage = 0;  // parity selects the halo buffer
    int wpar = 0;   // parity selects the weight buffer
    // Statistics: the tile whose per-wave channel sums wait in LDS to be added up and written (-1: none).  Every wave
    // writes its sums at the end of the tile's epilogue and goes on; the first 2 * WROWS threads add the 8 waves up
    // behind the next barrier that every wave has passed with its rows written.
    int pending_tile = -1, pending_count = 0;
    auto flush_sums = [&]() __attribute__((always_inline)) {
        if (tid < WROWS * 2) {
            const float* sred = reinterpret_cast<const float*>(lds + LD::SUMS_OFF);
            const int c = tid >> 1, k = tid & 1;
            float v = 0.f;
#pragma unroll
            for (int q = 0; q < 8; ++q) v += sred[q * 128 + c * 2 + k];
            a.part[((int64_t)pending_tile * a.Cout + co0 + c) * 2 + k] = v;
        }
        if (a.counts && tid == 0 && cbi == 0 && (walk || pending_tile < a.tiles_per_n)) a.counts[pending_tile] = pending_count;
        pending_tile = -1;
    };
    // The multiply pipeline: every column fetches the fragments of the next one, across groups, chunks and tiles.
    Frags<COB> fr;
    load_first<COB, 0, 0>(fr, hbuf0, wbuf0 + a_base, boff);
    constexpr int ROWB = LD::ROWB;                // padded row of the patch
    constexpr int PARTS = WROWS / 8;              // 16-byte parts per row: 8 or 4
    constexpr int RPI = 64 / PARTS;               // rows covered per read instruction
    // One 16-channel chunk = three tap groups; P = fragment slot of its first column (a group has an odd number of
    // columns / taps, so the slot alternates from group to group).
    auto chunk_groups = [&](f32x16 (&acc)[COB][NVB], int chunk, int tile, int next_tile, const HaloTile& ht_cur,
                            const HaloTile& ht_next) __attribute__((always_inline)) {
        constexpr int P = 0;
        const char* hb = hbuf0 + (stage & 1) * HALO_BYTES;
        char* hb_next = hbuf0 + ((stage + 1) & 1) * HALO_BYTES;
        const char* hbn = hb_next;
        // what streams in during this stage: the next chunk of this tile, or chunk 0 of the next
        const bool last_chunk = chunk + 1 == c_hi;
        const int pf_chunk = last_chunk ? c_lo : chunk + 1;
        const bool pf = !last_chunk || next_tile < tile_hi;
        const HaloTile ht = last_chunk ? ht_next : ht_cur;   // a copy: a reference picked at run time would put both in memory
        const char* w0p = wbuf0 + wpar * WBUF_BYTES + a_base;
        const char* w1p = wbuf0 + (wpar ^ 1) * WBUF_BYTES + a_base;
        const uint32_t hb_next_a = lds_a + ((stage + 1) & 1) * HALO_BYTES;
        const uint32_t w0n = wbuf_a + wpar * WBUF_BYTES, w1n = wbuf_a + (wpar ^ 1) * WBUF_BYTES;
        // weights copied behind the barriers of the three groups: group 2 of this chunk, groups 0 and 1 of the next
        const bf16_t* wc2 = wbase + (int64_t)chunk * (3 * wgstride) + 2 * wgstride;
        const bf16_t* wn0 = wbase + (int64_t)pf_chunk * (3 * wgstride);
        CopyCtx cc;
        cc.hb_next = hb_next; cc.hb_next_a = hb_next_a; cc.pf_halo = pf; cc.pf_choff = choff(pf_chunk); cc.zero16 = a.zero16;
        cc.abp = nullptr; cc.relu_floor = a.relu_floor; cc.wv = wv; cc.lane = lane;
        cc.tab = lds + LD::TAB_OFF; cc.tab_a = tab_a; cc.H = a.H; cc.W = a.W; cc.ldx = a.ldx;
        if constexpr (NORM) {
            const int n_pf = last_chunk && next_tile < tile_hi ? pos_next.n : pos.n;
            cc.abp = a.ab + (int64_t)n_pf * a.Cin + pf_chunk * 16;
        }
        cc.wb_fill_a = w0n; cc.pf_w = true; cc.wsrc = wc2;
        // (after group 0: every wave is past its barrier, its sums of the last tile written)
        conv_group<COB, TDT, 0, P, NORM>(acc, fr, hb, w0p, hb, w1p, boff, cc, hl, ht, wrel, ZERO_START && chunk == c_lo);
        if (pending_tile >= 0) flush_sums();
        cc.wb_fill_a = w1n; cc.pf_w = pf; cc.wsrc = wn0;
        conv_group<COB, TDT, 1, P ^ 1, NORM>(acc, fr, hb, w1p, hb, w0p, boff, cc, hl, ht, wrel);
        cc.wb_fill_a = w0n; cc.wsrc = wn0 + wgstride;
        conv_group<COB, TDT, 2, P, NORM>(acc, fr, hb, w0p, hbn, w1p, boff, cc, hl, ht, wrel);
        wpar ^= 1;
    };
    // The accumulators start a tile at zero.  32-channel block: the first column of a tile gives every accumulator's
    // first matrix instruction a zero addend (a second code path for that one column).  64-channel block: the
    // epilogue clears them as it hands each block on -- the second code path costs that kernel registers it has not got.
    f32x16 acc[COB][NVB];
#pragma unroll
    for (int cb = 0; cb < COB; ++cb)
#pragma unroll
        for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[cb][vb][r] = 0.f;
    for (; tile < tile_hi; tile += wg_per_xcd) {
        const int next_tile = tile + wg_per_xcd;
        TilePos pos_nn = pos;
        auto advance_pos = [&]() __attribute__((always_inline)) { pos_nn = tile_step(pos_next); };
        auto end_pass = [&]() __attribute__((always_inline)) {
            pos = pos_next;
            pos_next = pos_nn;
            ht_cur = ht_next;
            ht_next = halo_tile(pos_nn);
        };
        for (int chunk = c_lo; chunk < c_hi; ++chunk, ++stage) {
            chunk_groups(acc, chunk, tile, next_tile, ht_cur, ht_next);
            // a chunk has an odd number of columns: what its last column fetched sits in slot 1, and every chunk
            // starts in slot 0 (two code paths, one per starting slot, cost the compiler a hundred registers)
#pragma unroll
            for (int kd = 0; kd < 3; ++kd)
#pragma unroll
                for (int cb = 0; cb < COB; ++cb) fr.a[0][kd][cb] = fr.a[1][kd][cb];
        }
        const int n = pos.n, d0 = pos.d0, h0 = pos.h0, w0 = pos.w0;
        if constexpr (!LD::EPI_OWN) {
            // every wave has read its last fragments of the finished chunk's halo before any wave's epilogue writes there
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
        const int gd0 = d0 + ND * ds;
        if constexpr (SPLIT) {
            // fp32 partial sums straight from the accumulators: lane = voxel (bh, bw) of block vb, four
            // consecutive channels per register group
            static_assert(TDT == 4, "the split reduction uses the 4-deep tile");
            float* zp = a.zpart + (int64_t)blockIdx.z * ((int64_t)a.N * a.D * a.H * a.W) * a.Cout;
            if (a.bias && blockIdx.z == 0) {   // the first split's partial carries the bias
#pragma unroll
                for (int cb = 0; cb < COB; ++cb)
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        const float4 bv = *reinterpret_cast<const float4*>(a.bias + co0 + cb * 32 + rg * 8 + half * 4);
#pragma unroll
                        for (int vb = 0; vb < NVB; ++vb) {
                            acc[cb][vb][rg * 4 + 0] += bv.x; acc[cb][vb][rg * 4 + 1] += bv.y;
                            acc[cb][vb][rg * 4 + 2] += bv.z; acc[cb][vb][rg * 4 + 3] += bv.w;
                        }
                    }
            }
#pragma unroll
            for (int vb = 0; vb < NVB; ++vb) {
                const int gd = gd0 + vb, gh = h0 + hs + 4 * bh, gw = w0 + bw;
                if (gd < a.D && gh < a.H && gw < a.W) {
                    float* row = zp + ((((int64_t)n * a.D + gd) * a.H + gh) * a.W + gw) * a.Cout + co0 + half * 4;
#pragma unroll
                    for (int cb = 0; cb < COB; ++cb)
#pragma unroll
                        for (int rg = 0; rg < 4; ++rg)
                            *reinterpret_cast<float4*>(row + cb * 32 + rg * 8) =
                                make_float4(acc[cb][vb][rg * 4 + 0], acc[cb][vb][rg * 4 + 1], acc[cb][vb][rg * 4 + 2], acc[cb][vb][rg * 4 + 3]);
                }
                if constexpr (!ZERO_START) {
#pragma unroll
                    for (int cb = 0; cb < COB; ++cb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[cb][vb][r] = 0.f;
                }
            }
            advance_pos();
            end_pass();
            __syncthreads();
            continue;
        }
        // ---- epilogue.  Each wave turns its accumulators (lane = voxel, 4 consecutive channels per
        // register group) into voxel rows through a private LDS patch, so that 8 (4) lanes store one
        // full row of 64 (32) channels; the channel sums of the stored values come from the same pass.
        // Scratch: the patch region, or (64-channel block, 8-deep tile) the halo buffer of the stage just finished,
        // free until the next prefetch.
        char* fbuf = LD::EPI_OWN ? lds + LD::PATCH_OFF : hbuf0 + ((stage + 1) & 1) * HALO_BYTES;
        static_assert(LD::EPI_OWN || LD::PATCH_BYTES <= HALO_BYTES, "the patches fit the halo buffer");
        char* patch = fbuf + wv * (32 * ROWB);
        float* sred = reinterpret_cast<float*>(lds + LD::SUMS_OFF);
        // 64-channel block: the lane id enters the epilogue through an opaque copy, as what is derived from it below
        // would otherwise be hoisted out of the tile loop and stay in registers across the multiply loop, which has
        // none to spare.  The 32-channel block has them, and is the one whose epilogue weighs: there the hoisting is welcome.
        int lane_e = lane;
        if constexpr (COB == 2) asm volatile("" : "+v"(lane_e));
        const int part = lane_e % PARTS, prow = lane_e / PARTS;
        float csum[8], csq[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            csum[e] = WALK_OK ? ksum[WALK_OK ? e : 0] : 0.f;
            csq[e] = WALK_OK ? ksq[WALK_OK ? e : 0] : 0.f;
        }
        // Where this lane's 16-byte pieces go.  Its 8 channels, and with them the tensor and the channel
        // stride, are fixed; the tile origin is wave-uniform; what is left per store is a small offset
        // inside the tile.  Tiles that lie inside the volume (all but the ragged rim) skip the bounds tests.
        const int ch = co0 + part * 8;
        const bool second = ch >= a.zsplit;
        const int ldo = second ? a.ldz2 : a.ldz;
        const int hb0 = h0 + hs;
        bf16_t* const tbase = (second ? a.z2 + (ch - a.zsplit) : a.z + ch) +
                              ((((int64_t)n * a.D + gd0) * a.H + hb0) * a.W + w0) * ldo;
        const int vbvox = a.H * a.W;   // voxels from block vb to vb + 1 (offsets inside a tile fit 32 bits)
        // BSUM: the matching piece of the layer below's z (same offsets: same shape and channel stride), and this
        // lane's 8 (a, b) pairs
        const bf16_t* zbase = nullptr;
        float za[8], zbb[8];
        if constexpr (BSUM) {
            zbase = a.zb + ch + ((((int64_t)n * a.D + gd0) * a.H + hb0) * a.W + w0) * ldo;
            const float4* t = reinterpret_cast<const float4*>(a.zab + (int64_t)n * a.Cout + ch);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float4 v = t[e];
                za[2 * e] = v.x; zbb[2 * e] = v.y; za[2 * e + 1] = v.z; zbb[2 * e + 1] = v.w;
            }
        }
        const bool full = gd0 + ND <= a.D && h0 + TH <= a.H && w0 + TW <= a.W;
        const bool want_stats = a.part != nullptr;
        if (a.bias) {   // fp32 bias on the accumulators: what is rounded, stored and summed is z + b
#pragma unroll
            for (int cb = 0; cb < COB; ++cb)
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    const float4 bv = *reinterpret_cast<const float4*>(a.bias + co0 + cb * 32 + rg * 8 + half * 4);
#pragma unroll
                    for (int vb = 0; vb < NVB; ++vb) {
                        acc[cb][vb][rg * 4 + 0] += bv.x; acc[cb][vb][rg * 4 + 1] += bv.y;
                        acc[cb][vb][rg * 4 + 2] += bv.z; acc[cb][vb][rg * 4 + 3] += bv.w;
                    }
                }
        }
        // element offsets of this lane's rows inside a block (row = voxel index of the 32-voxel block, two h-rows 4 apart)
        int rowoff[32 / RPI];
#pragma unroll
        for (int i = 0; i < 32 / RPI; ++i) {
            const int row = prow + i * RPI, rg8 = row >> 3;
            rowoff[i] = (4 * ((rg8 ^ (rg8 >> 1)) & 1) * a.W + (row & 7) + 8 * (rg8 >> 1)) * ldo;
        }
        auto store_blocks = [&](auto FULLC) __attribute__((always_inline)) {
            constexpr bool FULL = decltype(FULLC)::value;
#pragma unroll
            for (int vb = 0; vb < NVB; ++vb) {
#pragma unroll
                for (int cb = 0; cb < COB; ++cb)
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        const uint32_t p0 = pack_bf16(acc[cb][vb][rg * 4 + 0], acc[cb][vb][rg * 4 + 1]);
                        const uint32_t p1 = pack_bf16(acc[cb][vb][rg * 4 + 2], acc[cb][vb][rg * 4 + 3]);
                        *reinterpret_cast<uint2*>(patch + l32 * ROWB + (cb * 32 + rg * 8 + half * 4) * 2) = make_uint2(p0, p1);
                        if constexpr (!ZERO_START) {
#pragma unroll
                            for (int r = 0; r < 4; ++r) acc[cb][vb][rg * 4 + r] = 0.f;
                        }
                    }
                __builtin_amdgcn_wave_barrier();
                if (vb == 0) advance_pos();   // scalar work in the shadow of the patch round trip
                bf16_t* const bbase = tbase + (int64_t)vb * vbvox * ldo;
                uint4 qv[32 / RPI];
                uint4 zv[BSUM ? 32 / RPI : 1];
#pragma unroll
                for (int i = 0; i < 32 / RPI; ++i) {
                    const int row = prow + i * RPI;          // voxel index inside the 32-voxel block
                    qv[i] = *reinterpret_cast<const uint4*>(patch + row * ROWB + part * 16);
                    bool ok = true;
                    if constexpr (!FULL) {
                        const int rg8 = row >> 3;
                        const int rw = (row & 7) + 8 * (rg8 >> 1), rh = 4 * ((rg8 ^ (rg8 >> 1)) & 1);
                        const int gd = gd0 + vb;
                        const int gh = hb0 + rh, gw = w0 + rw;
                        ok = gd < a.D && gh < a.H && gw < a.W;
                    }
                    if (ok) {
                        // streaming store: the output is not read again by this kernel and should not displace
                        // the input lines that the next chunk passes and the neighbouring tiles still need
                        typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
                        const u32x4 sv = {qv[i].x, qv[i].y, qv[i].z, qv[i].w};
                        __builtin_nontemporal_store(sv, reinterpret_cast<u32x4*>(bbase + rowoff[i]));
                        if constexpr (BSUM) zv[i] = *reinterpret_cast<const uint4*>(zbase + (int64_t)vb * vbvox * ldo + rowoff[i]);
                    } else {
                        qv[i] = make_uint4(0u, 0u, 0u, 0u);   // outside the volume: nothing stored, nothing summed
                        if constexpr (BSUM) zv[i] = make_uint4(0u, 0u, 0u, 0u);
                    }
                }
                if constexpr (BSUM) {
                    // sums of the InstanceNorm + ReLU backward below: g = [u > 0] * (stored value), (sum g, sum g*z)
#pragma unroll
                    for (int i = 0; i < 32 / RPI; ++i) {
                        const uint32_t r4[4] = {qv[i].x, qv[i].y, qv[i].z, qv[i].w}, z4[4] = {zv[i].x, zv[i].y, zv[i].z, zv[i].w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float z0 = __uint_as_float(z4[e] << 16), z1 = __uint_as_float(z4[e] & 0xFFFF0000u);
                            const float g0 = norm_u(z0, za[2 * e], zbb[2 * e]) > 0.f ? __uint_as_float(r4[e] << 16) : 0.f;
                            const float g1 = norm_u(z1, za[2 * e + 1], zbb[2 * e + 1]) > 0.f ? __uint_as_float(r4[e] & 0xFFFF0000u) : 0.f;
                            csum[2 * e] += g0; csq[2 * e] = fmaf(g0, z0, csq[2 * e]);
                            csum[2 * e + 1] += g1; csq[2 * e + 1] = fmaf(g1, z1, csq[2 * e + 1]);
                        }
                    }
                } else
                if (want_stats) {
                    // Sums of the stored (rounded) values, two voxels at a time: a byte permute puts the same channel
                    // of two voxels side by side, and one two-element dot product with (1, 1), one with the pair
                    // itself, add both voxels to the channel's sum and sum of squares (1.5 instead of 3 vector
                    // instructions per value).
                    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
                    const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3F803F80u);
#pragma unroll
                    for (int i = 0; i < 32 / RPI; i += 2) {
                        const uint32_t ra[4] = {qv[i].x, qv[i].y, qv[i].z, qv[i].w};
                        const uint32_t rb[4] = {qv[i + 1].x, qv[i + 1].y, qv[i + 1].z, qv[i + 1].w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const bf16x2 lo = __builtin_bit_cast(bf16x2, __builtin_amdgcn_perm(rb[e], ra[e], 0x05040100u));
                            const bf16x2 hi = __builtin_bit_cast(bf16x2, __builtin_amdgcn_perm(rb[e], ra[e], 0x07060302u));
                            csum[2 * e] = __builtin_amdgcn_fdot2_f32_bf16(lo, ones, csum[2 * e], false);
                            csq[2 * e] = __builtin_amdgcn_fdot2_f32_bf16(lo, lo, csq[2 * e], false);
                            csum[2 * e + 1] = __builtin_amdgcn_fdot2_f32_bf16(hi, ones, csum[2 * e + 1], false);
                            csq[2 * e + 1] = __builtin_amdgcn_fdot2_f32_bf16(hi, hi, csq[2 * e + 1], false);
                        }
                    }
                }
                __builtin_amdgcn_wave_barrier();
            }
        };
        if (full) store_blocks(std::true_type{});
        else store_blocks(std::false_type{});
        const int tile_count = min(TD, a.D - d0) * min(TH, a.H - h0) * min(TW, a.W - w0);
        bool fold_now = a.part != nullptr;
        if constexpr (WALK_OK) {
            wcount += tile_count;
            last_n = n;
            if (walk && next_tile < tile_hi && pos_next.n == n) {   // the walk goes on inside this sample
                fold_now = false;
#pragma unroll
                for (int e = 0; e < 8; ++e) { ksum[e] = csum[e]; ksq[e] = csq[e]; }
            }
        }
        if (fold_now) {
            // Lanes with equal `part` hold the same 8 channels.  Inside a row of 16 lanes they are folded by
            // rotations of the row (data-parallel primitives: no LDS traffic, where lane exchanges through the
            // LDS cost more than the tile's whole transpose); the 4 rows of a wave and the 8 waves are added by
            // the threads that write the tile's partial.
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                csum[e] += row_ror<8>(csum[e]);
                csq[e] += row_ror<8>(csq[e]);
                if constexpr (PARTS == 4) {
                    csum[e] += row_ror<4>(csum[e]);
                    csq[e] += row_ror<4>(csq[e]);
                }
            }
            // the wave's four lane rows meet in its own patch (free again), one (channel, sum kind) pair per lane and turn
            float* wrow = reinterpret_cast<float*>(patch);
            if ((lane_e & 15) < PARTS) {   // then part == lane & 15
                float* dst = wrow + ((lane_e >> 4) * 64 + part * 8) * 2;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    dst[2 * e + 0] = csum[e];
                    dst[2 * e + 1] = csq[e];
                }
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int t = 0; t < WROWS * 2 / 64; ++t) {
                const int ck = lane_e + 64 * t;
                sred[wv * 128 + ck] = (wrow[ck] + wrow[128 + ck]) + (wrow[256 + ck] + wrow[384 + ck]);
            }
            // No barrier: the sums are added up and written behind the first barrier of the next tile (after the
            // last tile: behind a barrier of their own), which every wave reaches with its rows written.
            pending_tile = walk ? n * a.walk_parts + walker : tile;
            pending_count = walk ? wcount : tile_count;
            if constexpr (WALK_OK) {
                wcount = 0;
#pragma unroll
                for (int e = 0; e < 8; ++e) { ksum[e] = 0.f; ksq[e] = 0.f; }
            }
        }
        end_pass();
        // No barrier here: the next copies into the patch buffer go out behind the barrier of the next tile's first
        // group.
    }
    if (pending_tile >= 0) {
        __builtin_amdgcn_s_waitcnt(0xC07F);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        flush_sums();
    }
    if constexpr (WALK_OK) {
        // the samples this walk holds no tile of
        if (walk && a.counts && tid == 0 && cbi == 0)
            for (int n = 0; n < a.N; ++n)
                if (n < first_n || n > last_n) a.counts[n * a.walk_parts + walker] = 0;
    }
}

// (a, b) of the normalise-on-load for every (sample, channel): u = a*x + b with the library's one formula.
__global__ __launch_bounds__(256) void norm_coeff_kernel(NormIn nm, int N, int C, float2* __restrict__ ab) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= N * C) return;
    float a, b;
    norm_coeffs(nm, i / C, i % C, a, b);
    ab[i] = make_float2(a, b);
}

static void tile_dims(const lamp_tensor_desc* t, int TD, int& td, int& th, int& tw) {
    td = (t->d + TD - 1) / TD; th = (t->h + TH - 1) / TH; tw = (t->w + TW - 1) / TW;
}

struct PackPlan { int gh, gw, hp, wp; };
static bool conv_pack_plan(const lamp_tensor_desc* zd, PackPlan& best);
static int conv_splits(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd);

bool mfma_conv_supported(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd, const lamp_norm_in* xnorm,
                         const float* bias) {
    if (xd->dtype != LAMP_BF16) return false;
    if (bias && (((uintptr_t)bias) & 15u)) return false;   // the epilogue reads it four floats at a time
    if (xd->c % 16 || zd->c % 32 || xd->ldc % 8 || zd->ldc % 8) return false;
    // element offsets inside a tile's halo (10 slices of H x W voxels) are kept in 32 bits
    const int64_t ldmax = xd->ldc > zd->ldc ? xd->ldc : zd->ldc;
    if ((int64_t)10 * zd->h * zd->w * ldmax >= ((int64_t)1 << 31)) return false;
    if (nvox(xd) >= ((int64_t)1 << 31)) return false;   // the voxel index of a tile's origin is kept in 32 bits
    // the halo copies' address arithmetic uses 24-bit multiplies
    if ((int64_t)10 * zd->h + 10 >= (1 << 24) || (int64_t)zd->w * xd->ldc >= (1 << 24)) return false;
    if (xnorm && xnorm->mean_rstd && xnorm->c_norm > 0) {
        // normalise on load: every input channel normalised, on the plain tiled kernel (no packed batch of tiny
        // volumes, no input-channel split: those layers are small and keep the generic path)
        PackPlan pp;
        if (xnorm->c_norm != xd->c || conv_pack_plan(zd, pp) || conv_splits(xd, zd) > 1) return false;
    }
    return true;
}

// Tile depth.  The 8-deep tile gives each wave a 128-voxel x 64-channel register tile (fewest LDS
// bytes and barriers per MFMA); the 4-deep tile yields twice the workgroup-tiles, which fills the chip
// on small volumes and wastes less of a last, partial round on medium ones.  (The 4-deep tile also halves the
// HBM re-fetch -- its per-XCD working set fits the 4 MiB L2 between chunk passes -- but is slower
// per MFMA.)  LAMP_TUNE=tile_depth=4|8 forces one.
static int conv_tile_depth(const lamp_tensor_desc* zd) {
    const int forced = tune("tile_depth", 0);
    if (forced == 4 || forced == 8) return forced;
    // Rounds of the chip: (tiles x output-channel blocks) workgroup-tiles over 256 CUs, rounded up; an 8-deep
    // tile costs 1.9 four-deep ones.  (Measured on 15 layer shapes from 32^3 to 176 x 128 x 144 with 32 to 256
    // channels: the cheaper side of this comparison was the faster kernel on every one.)
    const int64_t hw = (int64_t)zd->n * ((zd->h + TH - 1) / TH) * ((zd->w + TW - 1) / TW);
    const int64_t ncb = (zd->c + (zd->c % 64 == 0 ? 64 : 32) - 1) / (zd->c % 64 == 0 ? 64 : 32);
    const int64_t rounds8 = (hw * ((zd->d + 7) / 8) * ncb + 255) / 256, rounds4 = (hw * ((zd->d + 3) / 4) * ncb + 255) / 256;
    return 19 * rounds8 <= 10 * rounds4 ? 8 : 4;
}

// ---- many small volumes: one packed volume ---------------------------------------------------------
// A batch of tiny volumes (the deep levels of a batch of sliding windows) fills a 4 x 8 x 16 tile
// badly: a 4^3 sample uses 64 of its 512 voxel slots.  Such a batch is laid out as ONE volume
// [1][D][gh*(H+1)][gw*(W+1)]: sample n = a*gw + b sits at rows a*(H+1).. and columns b*(W+1)..,
// followed by one row / column of zeros, which is the zero padding of both neighbours.  The conv of
// the packed volume equals the per-sample conv at every real voxel; the voxels in the gaps are
// dropped when the result is copied back.
static int64_t pack_slots(int d, int h, int w) { return (int64_t)((d + 3) / 4) * ((h + TH - 1) / TH) * ((w + TW - 1) / TW); }
static bool conv_pack_plan(const lamp_tensor_desc* zd, PackPlan& best) {
    if (tune("no_pack", 0) || zd->n < 4 || zd->w > 8 || zd->h > 16 || zd->d > 64 || zd->c > 4096) return false;
    const int64_t plain = (int64_t)zd->n * pack_slots(zd->d, zd->h, zd->w);
    int64_t bs = plain;
    bool found = false;
    for (int gh = 1; gh <= 8 && gh <= zd->n; ++gh) {
        const int gw = (zd->n + gh - 1) / gh;
        const int hp = gh * (zd->h + 1), wp = gw * (zd->w + 1);
        const int64_t sl = pack_slots(zd->d, hp, wp);
        if ((int64_t)zd->d * hp * wp * 4096 >= ((int64_t)1 << 31)) continue;   // 32-bit element offsets, up to 4096 channels
        if (sl * 5 <= plain * 4 && sl < bs) { bs = sl; best = PackPlan{gh, gw, hp, wp}; found = true; }   // at least a fifth fewer tiles
    }
    return found;
}
static void pack_descs(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd, const PackPlan& p, lamp_tensor_desc& xp,
                       lamp_tensor_desc& zp) {
    xp = *xd; xp.n = 1; xp.h = p.hp; xp.w = p.wp; xp.ldc = xd->c;
    zp = *zd; zp.n = 1; zp.h = p.hp; zp.w = p.wp; zp.ldc = zd->c;
}

// One thread per (packed voxel, 16-byte granule of 8 channels).  Channels from csplit on come from x2.
__global__ __launch_bounds__(256) void conv_pack_kernel(const bf16_t* __restrict__ x, int ldx, const bf16_t* __restrict__ x2,
                                                        int csplit, bf16_t* __restrict__ xp, int N, int D, int H, int W, int C,
                                                        int gw, int hp, int wp) {
    const int gpv = C / 8;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)D * hp * wp * gpv) return;
    const int g = (int)(i % gpv);
    int64_t v = i / gpv;
    const int wq = (int)(v % wp); v /= wp;
    const int hq = (int)(v % hp);
    const int d = (int)(v / hp);
    const int a = hq / (H + 1), h = hq % (H + 1), b = wq / (W + 1), w = wq % (W + 1);
    const int n = a * gw + b;
    uint4 q = make_uint4(0, 0, 0, 0);
    if (h < H && w < W && n < N) {
        const int c = g * 8;
        const bf16_t* src = c < csplit ? x + c : x2 + (c - csplit);
        q = *reinterpret_cast<const uint4*>(src + ((((int64_t)n * D + d) * H + h) * W + w) * ldx);
    }
    *reinterpret_cast<uint4*>(xp + i * 8) = q;
}

// One workgroup per (sample, 64 output channels): copies the sample's voxels out of the packed result
// and, when stats != nullptr, takes mean and rstd of the stored values per channel (fixed order).
__global__ __launch_bounds__(256) void conv_unpack_kernel(const bf16_t* __restrict__ zp, bf16_t* __restrict__ z, int ldz, int N,
                                                          int D, int H, int W, int C, int gw, int hp, int wp, float eps,
                                                          float* __restrict__ stats) {
    __shared__ float red[2][32][64];
    const int n = blockIdx.x, c0 = blockIdx.y * 64;
    const int g = threadIdx.x & 7, vl = threadIdx.x >> 3;
    const int a = n / gw, b = n % gw;
    const int V = D * H * W;
    float s[8], q[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { s[e] = 0.f; q[e] = 0.f; }
    const int c = c0 + g * 8;
    if (c < C) {
        for (int v = vl; v < V; v += 32) {
            const int w = v % W, h = (v / W) % H, d = v / (W * H);
            const int64_t pv = ((int64_t)d * hp + a * (H + 1) + h) * wp + b * (W + 1) + w;
            const uint4 t = *reinterpret_cast<const uint4*>(zp + pv * C + c);
            *reinterpret_cast<uint4*>(z + ((((int64_t)n * D + d) * H + h) * W + w) * ldz + c) = t;
            const uint32_t r[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float f0 = __uint_as_float(r[e] << 16), f1 = __uint_as_float(r[e] & 0xFFFF0000u);
                s[2 * e] += f0; q[2 * e] = fmaf(f0, f0, q[2 * e]);
                s[2 * e + 1] += f1; q[2 * e + 1] = fmaf(f1, f1, q[2 * e + 1]);
            }
        }
    }
    if (!stats) return;
#pragma unroll
    for (int e = 0; e < 8; ++e) { red[0][vl][g * 8 + e] = s[e]; red[1][vl][g * 8 + e] = q[e]; }
    __syncthreads();
    if (threadIdx.x < 64 && c0 + (int)threadIdx.x < C) {
        double ss = 0.0, qq = 0.0;
        for (int r = 0; r < 32; ++r) { ss += (double)red[0][r][threadIdx.x]; qq += (double)red[1][r][threadIdx.x]; }
        const double mean = ss / V;
        double var = qq / V - mean * mean;
        if (var < 0.0) var = 0.0;
        float* o = stats + ((size_t)n * C + c0 + threadIdx.x) * 2;
        o[0] = (float)mean;
        o[1] = (float)(1.0 / sqrt(var + (double)eps));
    }
}

int conv_repack_kind(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd, bool two_out) {
    if (!mfma_conv_supported(xd, zd, nullptr, nullptr)) return -1;
    PackPlan pp;
    if (!two_out && conv_pack_plan(zd, pp)) {   // the conv runs on the packed volume, as one contiguous tensor
        lamp_tensor_desc xp, zp;
        pack_descs(xd, zd, pp, xp, zp);
        return conv_repack_kind(&xp, &zp, false);
    }
    return 1;   // one layout for both tile depths: tap groups by in-plane row kh
}
size_t conv_repack_bytes(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd) {
    return align_up((size_t)27 * xd->c * zd->c * 2 + 2 * xd->c + 64);
}

// Number of input-channel splits for the tiled kernel (1 = none): only where the 4-deep tiling with 64
// output channels per workgroup leaves at least half of the chip idle and there are chunks to share out.
static int conv_splits(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd) {
    if (tune("no_split", 0) || zd->c % 64 || conv_tile_depth(zd) != 4) return 1;
    int td, th, tw;
    tile_dims(zd, 4, td, th, tw);
    const int64_t wgs = (int64_t)zd->n * td * th * tw * (zd->c / 64);
    const int nchunks = xd->c / 16;
    if (wgs > 128 || nchunks < 8) return 1;   // measured: with 64 input channels the split costs more than it brings
    int S = (int)(256 / wgs);
    if (S > nchunks / 2) S = nchunks / 2;
    if (S < 2) return 1;
    const int cps = (nchunks + S - 1) / S;
    return (nchunks + cps - 1) / cps;
}

size_t mfma_conv_ws_bytes(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd, int want_stats) {
    if (!mfma_conv_supported(xd, zd, nullptr, nullptr)) return 0;
    const size_t ab_bytes = align_up((size_t)xd->n * xd->c * sizeof(float2));   // normalise-on-load coefficients
    int td, th, tw;
    tile_dims(zd, 4, td, th, tw);  // the finer tiling bounds the partial count
    const size_t tiles = (size_t)td * th * tw;
    // repacked weights + a run of zeros (source of the zero padding) + 16 bytes that absorb masked stores
    size_t b = align_up((size_t)27 * xd->c * zd->c * 2 + 2 * xd->c + 64);
    if (want_stats) {
        // partial statistics: one per tile, or one per (sample, workgroup walk) -- at most 256 walks
        const size_t parts = tiles > 256 ? tiles : 256;
        b += align_up((size_t)zd->n * parts * zd->c * 2 * sizeof(float)) + align_up((size_t)zd->n * parts * sizeof(int32_t));
    }
    const int S = conv_splits(xd, zd);
    if (S > 1) b += align_up((size_t)S * nvox(zd) * zd->c * sizeof(float)) + stats_ws_bytes(zd) + 256;
    PackPlan pp;
    if (conv_pack_plan(zd, pp)) {   // packed input and output + the inner conv's own workspace
        lamp_tensor_desc xp, zp;
        pack_descs(xd, zd, pp, xp, zp);
        const size_t pb = align_up((size_t)nvox(&xp) * xp.c * 2) + align_up((size_t)nvox(&zp) * zp.c * 2) +
                          mfma_conv_ws_bytes(&xp, &zp, 0) + 512;
        if (pb > b) b = pb;
    }
    return b + ab_bytes;
}

template <int COB, int TDT, bool SPLIT = false, bool NORM = false, bool BSUM = false>
static lamp_status launch_igemm(const ConvArgs& a, dim3 grid, hipStream_t s) {
    const int shm = Lds<TDT, COB>::LDS_BYTES;
    if (ensure_dyn_lds((const void*)conv3d_igemm_kernel<COB, TDT, SPLIT, NORM, BSUM>, shm) != LAMP_OK) return LAMP_ERR_HIP;
    hipLaunchKernelGGL((conv3d_igemm_kernel<COB, TDT, SPLIT, NORM, BSUM>), grid, dim3(512), shm, s, a);
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}

// The data gradient can carry the sums of the InstanceNorm backward below it where it runs on the plain tiled kernel
// and writes one tensor: no packed batch of tiny volumes, no input-channel split.
bool mfma_bsum_supported(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd) {
    if (tune("no_bsum", 0) || !mfma_conv_supported(xd, zd, nullptr, nullptr)) return false;
    PackPlan pp;
    return !conv_pack_plan(zd, pp) && conv_splits(xd, zd) == 1;
}
size_t mfma_bsum_ws_bytes(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd) {
    return mfma_conv_ws_bytes(xd, zd, 1) + align_up((size_t)zd->n * zd->c * sizeof(float2));
}

lamp_status mfma_conv_fwd(const lamp_tensor_desc* xd, const void* x, const void* w, bool dgrad,
                          const lamp_tensor_desc* zd, void* z, float* stats_out, float eps, void* ws, size_t ws_bytes,
                          hipStream_t s, const ConvParts* parts, const float* bias, const lamp_norm_in* xnorm,
                          const ConvBsum* bsum) {
    const bool two_in = parts && parts->x2, two_out = parts && parts->z2;
    const bool norm = xnorm && xnorm->mean_rstd && xnorm->c_norm > 0;
    if (norm && (two_in || !mfma_conv_supported(xd, zd, xnorm, bias))) return LAMP_ERR_UNSUPPORTED;
    if (bsum && (two_out || norm || stats_out || !mfma_bsum_supported(xd, zd) || (((uintptr_t)bsum->z) & 15u))) return LAMP_ERR_UNSUPPORTED;
    if (two_in && ((((uintptr_t)parts->x2) & 15u) || parts->x_c1 % 16 || parts->x_c1 <= 0 || parts->x_c1 >= xd->c)) return LAMP_ERR_ALIGN;
    if (two_out && ((((uintptr_t)parts->z2) & 15u) || parts->z_c1 % 32 || parts->z_c1 <= 0 || parts->z_c1 >= zd->c || parts->ldz2 % 8))
        return LAMP_ERR_ALIGN;
    if ((((uintptr_t)x) & 15u) || (((uintptr_t)z) & 15u) || (((uintptr_t)ws) & 15u) || (((uintptr_t)w) & 15u)) return LAMP_ERR_ALIGN;
    PackPlan pp;
    if (!two_out && conv_pack_plan(zd, pp)) {
        lamp_tensor_desc xp, zp;
        pack_descs(xd, zd, pp, xp, zp);
        Carver pc(ws, ws_bytes);
        bf16_t* xpk = (bf16_t*)pc.take((size_t)nvox(&xp) * xp.c * 2);
        bf16_t* zpk = (bf16_t*)pc.take((size_t)nvox(&zp) * zp.c * 2);
        const size_t inner = mfma_conv_ws_bytes(&xp, &zp, 0);
        void* iws = pc.take(inner);
        if (!pc.ok()) return LAMP_ERR_WORKSPACE;
        const int64_t granules = nvox(&xp) * (xp.c / 8);
        hipLaunchKernelGGL(conv_pack_kernel, dim3(cdiv(granules, 256)), dim3(256), 0, s, (const bf16_t*)x, xd->ldc,
                           two_in ? (const bf16_t*)parts->x2 : (const bf16_t*)x, two_in ? parts->x_c1 : xd->c, xpk, xd->n, xd->d,
                           xd->h, xd->w, xd->c, pp.gw, pp.hp, pp.wp);
        LAMP_CHECK_LAUNCH();
        lamp_status st = mfma_conv_fwd(&xp, xpk, w, dgrad, &zp, zpk, nullptr, 0.f, iws, inner, s, nullptr, bias);
        if (st != LAMP_OK) return st;
        hipLaunchKernelGGL(conv_unpack_kernel, dim3(zd->n, cdiv(zd->c, 64)), dim3(256), 0, s, zpk, (bf16_t*)z, zd->ldc, zd->n,
                           zd->d, zd->h, zd->w, zd->c, pp.gw, pp.hp, pp.wp, eps, stats_out);
        LAMP_CHECK_LAUNCH();
        return LAMP_OK;
    }
    const int TDT = conv_tile_depth(zd);
    int td, th, tw;
    tile_dims(zd, TDT, td, th, tw);
    const int tiles_per_n = td * th * tw;
    Carver cv(ws, ws_bytes);
    bf16_t* wp = (bf16_t*)cv.take((size_t)27 * xd->c * zd->c * 2 + 16);
    float* part = nullptr;
    int32_t* counts = nullptr;
    // one persistent workgroup per CU (LDS-limited), 32 per XCD; fewer where there are fewer tiles
    int wgx = 256;
    while (wgx > 8 && (wgx / 8) > (tiles_per_n * zd->n + 7) / 8) wgx -= 8;
    // statistics per walk: 32-channel block, at least four tiles to a walk (below that the per-tile partials are as few)
    const bool walk = stats_out && !bsum && zd->c % 64 != 0 && conv_splits(xd, zd) == 1 && !tune("no_walk_stats", 0) &&
                      (int64_t)tiles_per_n * zd->n >= 4 * wgx;
    if (stats_out) {
        const size_t parts = walk ? (size_t)wgx : (size_t)tiles_per_n;
        part = (float*)cv.take((size_t)zd->n * parts * zd->c * 2 * sizeof(float));
        counts = (int32_t*)cv.take((walk ? (size_t)zd->n * wgx : (size_t)tiles_per_n) * sizeof(int32_t));
    }
    float2* ab = nullptr;
    if (norm) ab = (float2*)cv.take((size_t)xd->n * xd->c * sizeof(float2));
    if (bsum) {   // per-tile partial sums, and the (a, b) table of the layer below (over this launch's output channels)
        part = (float*)cv.take((size_t)zd->n * tiles_per_n * zd->c * 2 * sizeof(float));
        ab = (float2*)cv.take((size_t)zd->n * zd->c * sizeof(float2));
    }
    if (!cv.ok()) return LAMP_ERR_WORKSPACE;
    if (bsum) {
        lamp_norm_in nb{bsum->stats, bsum->gamma, bsum->beta, zd->c, 1};
        hipLaunchKernelGGL(norm_coeff_kernel, dim3(cdiv((int64_t)zd->n * zd->c, 256)), dim3(256), 0, s, make_norm(&nb), zd->n, zd->c, ab);
        LAMP_CHECK_LAUNCH();
    }
    if (norm) {
        hipLaunchKernelGGL(norm_coeff_kernel, dim3(cdiv((int64_t)xd->n * xd->c, 256)), dim3(256), 0, s, make_norm(xnorm), xd->n, xd->c, ab);
        LAMP_CHECK_LAUNCH();
    }
    const int64_t wtotal = (int64_t)27 * xd->c * zd->c;
    if (const bf16_t* pre = find_prepacked(w, dgrad, 1, zd->c, xd->c)) {
        wp = const_cast<bf16_t*>(pre);
    } else {
        hipLaunchKernelGGL(repack_weights_kernel, dim3(cdiv(wtotal / 8, 256)), dim3(256), 0, s, (const bf16_t*)w, wp, zd->c, xd->c,
                           dgrad ? 1 : 0, 1);
        LAMP_CHECK_LAUNCH();
    }
    ConvArgs a;
    a.x = (const bf16_t*)x; a.ldx = xd->ldc; a.wp = wp; a.z = (bf16_t*)z; a.ldz = zd->ldc; a.part = part; a.counts = counts;
    a.zero16 = wp + (size_t)27 * xd->c * zd->c;
    a.bias = bias;
    a.ab = norm ? ab : nullptr;
    a.zb = bsum ? (const bf16_t*)bsum->z : nullptr;
    a.zab = bsum ? ab : nullptr;
    a.relu_floor = norm && !xnorm->relu ? -__builtin_inff() : 0.f;
    a.N = zd->n; a.D = zd->d; a.H = zd->h; a.W = zd->w; a.Cin = xd->c; a.Cout = zd->c;
    a.tiles_d = td; a.tiles_h = th; a.tiles_w = tw; a.tiles_per_n = tiles_per_n;
    a.tiles_total = tiles_per_n * zd->n;
    a.tiles_per_xcd = (a.tiles_total + 7) / 8;
    const int cob = (zd->c % 64 == 0) ? 2 : 1;
    a.walk_parts = walk ? wgx : 0;
    dim3 grid(wgx, zd->c / (32 * cob));
    a.zpart = nullptr; a.cps = 0;
    a.xcd_rot = a.tiles_total < 32 ? 1 : 0;
    a.cb_inner = 0;
    a.xdelta = two_in ? (int64_t)((const bf16_t*)parts->x2 - (const bf16_t*)x) : 0;
    a.xsplit = two_in ? parts->x_c1 / 16 : 0x7fffffff;
    a.z2 = two_out ? (bf16_t*)parts->z2 : nullptr;
    a.ldz2 = two_out ? parts->ldz2 : 0;
    a.zsplit = two_out ? parts->z_c1 : 0x7fffffff;
    const int S = conv_splits(xd, zd);
    if (S > 1) {
        a.zpart = (float*)cv.take((size_t)S * nvox(zd) * zd->c * sizeof(float));
        void* sws = cv.take(stats_ws_bytes(zd));
        if (!cv.ok()) return LAMP_ERR_WORKSPACE;
        a.cps = ((xd->c / 16) + S - 1) / S;
        a.part = nullptr; a.counts = nullptr;
        grid.z = S;
        lamp_status st = launch_igemm<2, 4, true>(a, grid, s);
        if (st != LAMP_OK) return st;
        return launch_splitk_reduce(a.zpart, S, zd, z, eps, stats_out, sws, stats_ws_bytes(zd), s, a.z2, a.ldz2, a.zsplit);
    }
    if (!a.xcd_rot && grid.y > 1 && !tune("cb_outer", 0)) {
        a.cb_inner = (int)grid.y;
        grid.x *= grid.y;
        grid.y = 1;
    }
    lamp_status st;
    if (bsum) {
        if (TDT == 8) st = cob == 2 ? launch_igemm<2, 8, false, false, true>(a, grid, s) : launch_igemm<1, 8, false, false, true>(a, grid, s);
        else st = cob == 2 ? launch_igemm<2, 4, false, false, true>(a, grid, s) : launch_igemm<1, 4, false, false, true>(a, grid, s);
        if (st != LAMP_OK) return st;
        return launch_bsum_finalize(part, tiles_per_n, zd->n, zd->c, bsum->stats, bsum->sums_out, s);
    }
    if (norm) {
        if (TDT == 8) st = cob == 2 ? launch_igemm<2, 8, false, true>(a, grid, s) : launch_igemm<1, 8, false, true>(a, grid, s);
        else st = cob == 2 ? launch_igemm<2, 4, false, true>(a, grid, s) : launch_igemm<1, 4, false, true>(a, grid, s);
    } else if (TDT == 8) st = cob == 2 ? launch_igemm<2, 8>(a, grid, s) : launch_igemm<1, 8>(a, grid, s);
    else st = cob == 2 ? launch_igemm<2, 4>(a, grid, s) : launch_igemm<1, 4>(a, grid, s);
    if (st != LAMP_OK) return st;
    if (stats_out) return launch_stats_finalize(part, counts, walk ? wgx : tiles_per_n, zd->n, zd->c, eps, stats_out, s, walk);
    return LAMP_OK;
}

// ------------------------------------------------------------------------------------------------
// Weight gradient:  dW[co][tap][ci] = sum_v dz[v][co] * x[v + tap][ci]
//
// GEMM view: M = co (A = dz^T), N = ci (B = x shifted by the tap), K = voxels.  Both operands are
// needed K-major per lane but live channel-major (NDHWC) in LDS, so fragments are read with the
// transposing LDS load (ds_read_b64_tr_b16): inside each 16-lane group, source lane s supplies
// 4 channels of voxel row s/4 and lane t receives channel t of 4 consecutive voxel rows.
// A workgroup (8 waves) owns one 32-wide ci block and 32*COB output channels for all 27 taps, a
// tap column (kd, kw) per wave plus one tap of the ninth column for three of them (<= 4 taps each,
// accumulators 2*4*16 registers), and walks a
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
    const bf16_t* zero16;  // 16 zero bytes in global memory
    int N, D, H, W, Cin, Cout;
    int tiles_d, tiles_h, tiles_w, tiles_per_n, tiles_total, tiles_per_wg;
    const bf16_t* x2; int xsplit;   // two-part x: input channels from xsplit on live in x2 (same channel stride)
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

// Per-lane constants of the wgrad tile copies (register-free global -> LDS, 16 voxels x 64 bytes per
// wave copy: lane = voxel*4 + 16-byte part).
//   dz: 2*COB/2... one copy = 16 voxels of one 32-channel half; x: 16 halo voxels of the 32-ci block.
struct WgradLane {
    int xrel[6];   // element offset of this lane's x halo voxel from the tile's halo origin, per copy slot
    int xpk[6];    // its halo coords (d | h<<8 | w<<16), or -1 when the slot has no voxel for this lane
    int zrel[4];   // element offset of this lane's dz voxel from the tile origin, per copy slot
    int zpk[4];    // its tile coords
};

// Fragment registers that live from one k-step to the next, and from a tile's last k-step to the first of the next tile.
template <int COB> struct WFrags {
    bf16x8 af[2][COB];   // dz fragments of a k-step, two slots
    bf16x8 rb[6];        // x row fragments of the wave's tap column, a ring of six register sets
    bf16x8 eb[2];        // x fragments of the extra tap (waves 0..2), two slots
};

// The fragments of k-step 0 of the tile in stage st: dz into slot 0, the first three rows into sets R0, R0+1, R0+2.
template <int COB, int NT, int R0>
__device__ __forceinline__ void wgrad_first(WFrags<COB>& f, const char* __restrict__ st, uint32_t coloff, uint32_t extoff, uint32_t loff) {
    const char* xb = st + loff + coloff;
#pragma unroll
    for (int cb = 0; cb < COB; ++cb) f.af[0][cb] = lds_frag_tr(st + WX_BYTES + loff + cb * WDZ_HALF_BYTES);
#pragma unroll
    for (int r = 0; r < 3; ++r) f.rb[R0 + r] = lds_frag_tr(xb + (uint32_t)(r * WHW * 64));
    if constexpr (NT == 4) f.eb[0] = lds_frag_tr(st + loff + extoff);
}

// One tile: 16 k-steps (one 16-voxel w-row of the tile each), with the copies of the next tile going out one or two
// per k-step behind the first ones (in one burst they hold the wave up while they queue).
// A wave owns one tap column (kd, kw) with its three taps kh = 0, 1, 2: at k-step (d, h) they read the x rows
// h, h+1, h+2 of halo slice d + kd, so from one k-step to the next two of the three row fragments stay in
// registers and one new row is read (three at the change of d): 20 row fragments per tile feed 48*COB matrix
// instructions, where a fragment per tap and k-step would be 48.  The ninth column (2, 2) has no wave of its
// own: waves 0, 1, 2 take one of its taps each (NT == 4), one more row fragment per k-step.
// Every k-step fetches the fragments of the next one, the last k-step those of the next tile's first: the workgroup's
// barrier sits before the last k-step, whose operands are in registers by then, so the matrix instructions behind the
// barrier start at once.  (At that barrier every wave has read the last fragments of this stage, which the copies
// issued from the next tile on may overwrite, and has seen its own copies of the next tile land.)
template <int COB, int NT>
__device__ __forceinline__ void wgrad_tile(f32x16 (&acc)[COB][4], WFrags<COB>& f, const char* __restrict__ st,
                                           char* __restrict__ st_next, bool pf, const WgradLane& wl, const bf16_t* xorg,
                                           const bf16_t* zorg, int dlo, int dhi, int hlo, int hhi, int wlo, int whi, int zd,
                                           int zh, int zw, const bf16_t* zero16, uint32_t coloff, uint32_t extoff, uint32_t loff,
                                           int wv) {
    constexpr int XCOPIES = WX_VOX / 16;            // 45
    constexpr int ZCOPIES = COB * WTILE_VOX / 16;   // 32 or 16
    // copy i of the x halo (q = wv + 8*i covers halo voxels 16q..16q+15) and of dz (half q / 16, voxels 16*(q%16) .. +15)
    auto copy_x = [&](int i) __attribute__((always_inline)) {
        const int q = wv + 8 * i;
        if (q < XCOPIES) {
            const int pk = wl.xpk[i];
            const int hd = pk & 255, hh = (pk >> 8) & 255, hw = pk >> 16;
            const bool in = hd >= dlo && hd <= dhi && hh >= hlo && hh <= hhi && hw >= wlo && hw <= whi;
            g2lds16(in ? xorg + wl.xrel[i] : zero16, st_next + q * 1024);
        }
    };
    auto copy_z = [&](int i) __attribute__((always_inline)) {
        const int q = wv + 8 * i;
        const int pk = wl.zpk[i];
        const int d = pk & 255, h = (pk >> 8) & 255, w = pk >> 16;
        const bool in = d < zd && h < zh && w < zw;
        g2lds16(in ? zorg + wl.zrel[i] : zero16, st_next + WX_BYTES + q * 1024);
    };
    const char* xb = st + loff + coloff;
    const char* xe = st + loff + extoff;
    const char* dzb = st + WX_BYTES + loff;
    // Row fragments of the column as one stream q = 10*d + r (r = halo row of slice d + kd); fragment q lives in
    // register set q % 6, which its predecessor q - 6 has left two k-steps earlier.  Everything a k-step needs is
    // read during the k-step before it.
    auto row = [&](int q) __attribute__((always_inline)) {
        return lds_frag_tr(xb + (uint32_t)(((q / 10) * WHH + (q % 10)) * WHW * 64));
    };
    auto ext = [&](int ks) __attribute__((always_inline)) {
        return lds_frag_tr(xe + (uint32_t)(((ks >> 3) * WHH + (ks & 7)) * WHW * 64));
    };
    auto load_a = [&](int ks, int slot) __attribute__((always_inline)) {
#pragma unroll
        for (int cb = 0; cb < COB; ++cb) f.af[slot][cb] = lds_frag_tr(dzb + cb * WDZ_HALF_BYTES + ks * 16 * 64);
    };
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {
        const int q0 = 10 * (ks >> 3) + (ks & 7);
        if (ks == 15) {
            // the copies of the next tile have landed, for every wave, and nobody reads this stage any more
            wait_vmcnt<0>();
            __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0), as a builtin so the compiler knows the reads are done
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            // first fragments of the next tile: k-step 15 multiplies with row sets 5, 0, 1, so the three rows go to
            // sets 2, 3, 4 and move to 0, 1, 2 behind it
            wgrad_first<COB, NT, 2>(f, st_next, coloff, extoff, loff);
        } else {
            load_a(ks + 1, (ks + 1) & 1);
            const int qn = 10 * ((ks + 1) >> 3) + ((ks + 1) & 7);
            if (((ks + 1) & 7) == 0) {   // next slice: three new rows
                f.rb[qn % 6] = row(qn);
                f.rb[(qn + 1) % 6] = row(qn + 1);
            }
            f.rb[(qn + 2) % 6] = row(qn + 2);
            if constexpr (NT == 4) f.eb[(ks + 1) & 1] = ext(ks + 1);
        }
#pragma unroll
        for (int kh = 0; kh < 3; ++kh)
#pragma unroll
            for (int cb = 0; cb < COB; ++cb)
                acc[cb][kh] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.af[ks & 1][cb], f.rb[(q0 + kh) % 6], acc[cb][kh], 0, 0, 0);
        if constexpr (NT == 4) {
#pragma unroll
            for (int cb = 0; cb < COB; ++cb)
                acc[cb][3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.af[ks & 1][cb], f.eb[ks & 1], acc[cb][3], 0, 0, 0);
        }
        constexpr int NM = NT * COB;   // MFMAs per k-step
        if (ks == 15 || ((ks + 1) & 7) == 0) sched_interleave<0, NM, 2 * (COB + 3 + (NT == 4 ? 1 : 0))>();
        else sched_interleave<0, NM, 2 * (COB + 1 + (NT == 4 ? 1 : 0))>();
        if (ks < 6) {   // this k-step's share of the next tile's copies: x copies 0..5, dz copies 0..3 (0..1)
            __builtin_amdgcn_sched_barrier(0);
            if (pf) {
                copy_x(ks);
                if (ks < ZCOPIES / 8) copy_z(ks);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    f.rb[0] = f.rb[2];
    f.rb[1] = f.rb[3];
    f.rb[2] = f.rb[4];
}

template <int COB>
__global__ __launch_bounds__(512) void conv3d_wgrad_kernel(WgradArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int ci0 = blockIdx.y * 32, co0 = blockIdx.z * (32 * COB);
    const bf16_t* xpart = ci0 < a.xsplit ? a.x + ci0 : a.x2 + (ci0 - a.xsplit);   // this workgroup's 32 input channels
    const int tile_lo = blockIdx.x * a.tiles_per_wg;
    const int tile_hi = min(tile_lo + a.tiles_per_wg, a.tiles_total);

    // taps of this wave: the column (kd, kw) = (wv / 3, wv % 3) with kh = 0, 1, 2 (accumulators 0..2); waves 0..2
    // also take tap (2, kh = wv, 2) of the ninth column (accumulator 3)
    const int col_kd = wv / 3, col_kw = wv % 3;
    const uint32_t coloff = (uint32_t)((col_kd * WHH * WHW + col_kw) * 64);
    const uint32_t extoff = (uint32_t)(((2 * WHH + wv) * WHW + 2) * 64);
    const bool has4 = wv < 3;

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

    // ---- per-lane constants of the tile copies
    WgradLane wl;
    const int cv = lane >> 2, cp = lane & 3;   // voxel within the copy, 16-byte part
#pragma unroll
    for (int i = 0; i < 6; ++i) {
        int hv = (wv + 8 * i) * 16 + cv;
        if (hv >= WX_VOX) hv = 0;
        const int hw = hv % WHW, hh = (hv / WHW) % WHH, hd = hv / (WHW * WHH);
        wl.xrel[i] = ((hd * a.H + hh) * a.W + hw) * a.ldx + cp * 8;
        wl.xpk[i] = hd | (hh << 8) | (hw << 16);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int q = wv + 8 * i;
        const int hf = q / 16, vx = (q % 16) * 16 + cv;   // (for COB == 1 only q < 16 is used: hf = 0)
        const int w = vx % WTW, h = (vx / WTW) % WTH, d = vx / (WTW * WTH);
        wl.zrel[i] = ((d * a.H + h) * a.W + w) * a.lddz + hf * 32 + cp * 8;
        wl.zpk[i] = d | (h << 8) | (w << 16);
    }
    // tiles are numbered d-fastest: consecutive tiles of a workgroup's walk share two of their four halo
    // d-slices, which the second one then finds in the XCD's L2
    auto tile_coords = [&](int tile, int& n, int& d0, int& h0, int& w0) {
        n = tile / a.tiles_per_n;
        int r = tile - n * a.tiles_per_n;
        d0 = (r % a.tiles_d) * WTD;
        r /= a.tiles_d;
        w0 = (r % a.tiles_w) * WTW;
        h0 = (r / a.tiles_w) * WTH;
    };

    WFrags<COB> fr;
    // one tile's copies + multiply; `cur` selects the LDS stage holding `tile`
    // (the position of the tile to fetch is stepped, not divided out, from tile to tile: the walk is contiguous)
    int fn, fd0, fh0, fw0;
    tile_coords(tile_lo, fn, fd0, fh0, fw0);
    const int lim_d = a.tiles_d * WTD, lim_w = a.tiles_w * WTW, lim_h = a.tiles_h * WTH;
    auto step_tile = [&]() __attribute__((always_inline)) {
        fd0 += WTD;
        if (fd0 >= lim_d) {
            fd0 = 0;
            fw0 += WTW;
            if (fw0 >= lim_w) {
                fw0 = 0;
                fh0 += WTH;
                if (fh0 >= lim_h) { fh0 = 0; ++fn; }
            }
        }
    };
    auto run_tile = [&](bool pf, const char* st, char* st_next) {
        const int n = fn, d0 = fd0, h0 = fh0, w0 = fw0;
        // (voxel indices fit 32 bits: checked on the host)
        const bf16_t* xorg = xpart + (int64_t)(((n * a.D + (d0 - 1)) * a.H + (h0 - 1)) * a.W + (w0 - 1)) * a.ldx;
        const bf16_t* zorg = a.dz + (int64_t)(((n * a.D + d0) * a.H + h0) * a.W + w0) * a.lddz + co0;
        if (has4)
            wgrad_tile<COB, 4>(acc, fr, st, st_next, pf, wl, xorg, zorg, 1 - d0, a.D - d0, 1 - h0, a.H - h0, 1 - w0, a.W - w0,
                               a.D - d0, a.H - h0, a.W - w0, a.zero16, coloff, extoff, loff, wv);
        else
            wgrad_tile<COB, 3>(acc, fr, st, st_next, pf, wl, xorg, zorg, 1 - d0, a.D - d0, 1 - h0, a.H - h0, 1 - w0, a.W - w0,
                               a.D - d0, a.H - h0, a.W - w0, a.zero16, coloff, extoff, loff, wv);
    };

    if (tile_lo < tile_hi) {
        // prologue: fetch the first tile into stage 0 (the multiply part runs on zero-filled... no:
        // only the copies are wanted here, so issue them directly)
        int n, d0, h0, w0;
        tile_coords(tile_lo, n, d0, h0, w0);
        const bf16_t* xorg = xpart + ((((int64_t)n * a.D + (d0 - 1)) * a.H + (h0 - 1)) * a.W + (w0 - 1)) * a.ldx;
        const bf16_t* zorg = a.dz + ((((int64_t)n * a.D + d0) * a.H + h0) * a.W + w0) * a.lddz + co0;
#pragma unroll
        for (int i = 0; i < 6; ++i) {
            const int q = wv + 8 * i;
            if (q < WX_VOX / 16) {
                const int pk = wl.xpk[i];
                const int hd = pk & 255, hh = (pk >> 8) & 255, hw = pk >> 16;
                const bool in = hd >= 1 - d0 && hd <= a.D - d0 && hh >= 1 - h0 && hh <= a.H - h0 && hw >= 1 - w0 && hw <= a.W - w0;
                g2lds16(in ? xorg + wl.xrel[i] : a.zero16, lds + q * 1024);
            }
        }
#pragma unroll
        for (int i = 0; i < COB * WTILE_VOX / 128; ++i) {
            const int q = wv + 8 * i;
            const int pk = wl.zpk[i];
            const bool in = (pk & 255) < a.D - d0 && ((pk >> 8) & 255) < a.H - h0 && (pk >> 16) < a.W - w0;
            g2lds16(in ? zorg + wl.zrel[i] : a.zero16, lds + WX_BYTES + q * 1024);
        }
    }
    wait_vmcnt<0>();
    __syncthreads();
    if (has4) wgrad_first<COB, 4, 0>(fr, lds, coloff, extoff, loff);
    else wgrad_first<COB, 3, 0>(fr, lds, coloff, extoff, loff);

    int par = 0;
    for (int tile = tile_lo; tile < tile_hi; ++tile, par ^= 1) {
        const bool pf = tile + 1 < tile_hi;
        if (pf) step_tile();
        run_tile(pf, lds + par * WBUF_STAGE, lds + (par ^ 1) * WBUF_STAGE);
    }

    // ---- write this workgroup's partial: part[slot][co][tap][ci]
    float* pb = a.part + (int64_t)blockIdx.x * a.Cout * 27 * a.Cin;
    const int l32 = lane & 31, half = lane >> 5;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = i < 3 ? col_kd * 9 + i * 3 + col_kw : 18 + wv * 3 + 2;
        if (i < 3 || has4) {
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
    // element offsets inside a tile's halo (4 slices of H x W voxels) are kept in 32 bits
    const int64_t ldmax = xd->ldc > dzd->ldc ? xd->ldc : dzd->ldc;
    if ((int64_t)4 * xd->h * xd->w * ldmax + 4096 >= ((int64_t)1 << 31)) return false;
    if (nvox(xd) >= ((int64_t)1 << 31)) return false;   // the voxel index of a tile's origin is kept in 32 bits
    return true;
}

// A batch of tiny volumes is laid out as one volume with a row / column of zeros between the samples, like the
// forward and data-gradient passes do (conv_pack_plan): the zeros are both neighbours' padding in x and contribute
// nothing in dz, so the weight gradient of the packed pair is the sum of the samples' weight gradients, over far fewer,
// fuller tiles.
static bool wgrad_pack_plan(const lamp_tensor_desc* xd, const lamp_tensor_desc* dzd, PackPlan& pp) {
    return xd->c % 8 == 0 && dzd->c % 8 == 0 && conv_pack_plan(dzd, pp);
}
size_t mfma_wgrad_ws_bytes(const lamp_tensor_desc* xd, const lamp_tensor_desc* dzd) {
    if (!mfma_wgrad_supported(xd, dzd, nullptr)) return 0;
    PackPlan pp;
    if (wgrad_pack_plan(xd, dzd, pp)) {
        lamp_tensor_desc xp, zp;
        pack_descs(xd, dzd, pp, xp, zp);
        return align_up((size_t)nvox(&xp) * xp.c * 2) + align_up((size_t)nvox(&zp) * zp.c * 2) + mfma_wgrad_ws_bytes(&xp, &zp) + 512;
    }
    return align_up((size_t)wgrad_slots(xd, dzd) * dzd->c * 27 * xd->c * sizeof(float)) + 256;
}


lamp_status mfma_wgrad(const lamp_tensor_desc* xd, const void* x, const lamp_tensor_desc* dzd, const void* dz, float* dw,
                       float beta, void* ws, size_t ws_bytes, hipStream_t s, const void* x2, int x_c1) {
    if ((((uintptr_t)x) & 15u) || (((uintptr_t)dz) & 15u) || (((uintptr_t)ws) & 15u)) return LAMP_ERR_ALIGN;
    if (x2 && ((((uintptr_t)x2) & 15u) || x_c1 % 32 || x_c1 <= 0 || x_c1 >= xd->c)) return LAMP_ERR_ALIGN;
    if (ws_bytes < mfma_wgrad_ws_bytes(xd, dzd)) return LAMP_ERR_WORKSPACE;
    PackPlan pp;
    if (wgrad_pack_plan(xd, dzd, pp)) {
        lamp_tensor_desc xp, zp;
        pack_descs(xd, dzd, pp, xp, zp);
        Carver pc(ws, ws_bytes);
        bf16_t* xpk = (bf16_t*)pc.take((size_t)nvox(&xp) * xp.c * 2);
        bf16_t* zpk = (bf16_t*)pc.take((size_t)nvox(&zp) * zp.c * 2);
        const size_t inner = mfma_wgrad_ws_bytes(&xp, &zp);
        void* iws = pc.take(inner);
        if (!pc.ok()) return LAMP_ERR_WORKSPACE;
        const int64_t gx = nvox(&xp) * (xp.c / 8), gz = nvox(&zp) * (zp.c / 8);
        hipLaunchKernelGGL(conv_pack_kernel, dim3(cdiv(gx, 256)), dim3(256), 0, s, (const bf16_t*)x, xd->ldc,
                           x2 ? (const bf16_t*)x2 : (const bf16_t*)x, x2 ? x_c1 : xd->c, xpk, xd->n, xd->d, xd->h, xd->w, xd->c,
                           pp.gw, pp.hp, pp.wp);
        LAMP_CHECK_LAUNCH();
        hipLaunchKernelGGL(conv_pack_kernel, dim3(cdiv(gz, 256)), dim3(256), 0, s, (const bf16_t*)dz, dzd->ldc, (const bf16_t*)dz,
                           dzd->c, zpk, dzd->n, dzd->d, dzd->h, dzd->w, dzd->c, pp.gw, pp.hp, pp.wp);
        LAMP_CHECK_LAUNCH();
        return mfma_wgrad(&xp, xpk, &zp, zpk, dw, beta, iws, inner, s, nullptr, 0);
    }
    WgradArgs a;
    a.x = (const bf16_t*)x; a.ldx = xd->ldc; a.dz = (const bf16_t*)dz; a.lddz = dzd->ldc; a.part = (float*)ws;
    a.x2 = (const bf16_t*)x2; a.xsplit = x2 ? x_c1 : 0x7fffffff;
    a.N = xd->n; a.D = xd->d; a.H = xd->h; a.W = xd->w; a.Cin = xd->c; a.Cout = dzd->c;
    wtile_dims(xd, a.tiles_d, a.tiles_h, a.tiles_w);
    a.tiles_per_n = a.tiles_d * a.tiles_h * a.tiles_w;
    a.tiles_total = a.tiles_per_n * xd->n;
    const int S = wgrad_slots(xd, dzd);
    a.tiles_per_wg = (a.tiles_total + S - 1) / S;
    // one slot and nothing to accumulate onto: the only partial IS the result (wide layers on small volumes,
    // whose dW runs to hundreds of megabytes), so the kernel writes it in place and no second pass is needed
    const bool direct = S == 1 && beta == 0.f;
    if (direct) a.part = dw;
    a.zero16 = device_zero16();
    if (!a.zero16) return LAMP_ERR_HIP;
    const int cob = (dzd->c % 64 == 0) ? 2 : 1;
    dim3 grid(S, xd->c / 32, dzd->c / (32 * cob));
    if (cob == 2) {
        if (ensure_dyn_lds((const void*)conv3d_wgrad_kernel<2>, WG_LDS_BYTES) != LAMP_OK) return LAMP_ERR_HIP;
        hipLaunchKernelGGL((conv3d_wgrad_kernel<2>), grid, dim3(512), WG_LDS_BYTES, s, a);
    } else {
        if (ensure_dyn_lds((const void*)conv3d_wgrad_kernel<1>, WG_LDS_BYTES) != LAMP_OK) return LAMP_ERR_HIP;
        hipLaunchKernelGGL((conv3d_wgrad_kernel<1>), grid, dim3(512), WG_LDS_BYTES, s, a);
    }
    LAMP_CHECK_LAUNCH();
    if (direct) return LAMP_OK;
    return launch_reduce_partials((const float*)ws, S, (int64_t)dzd->c * 27 * xd->c, dw, beta, s);
}

}  // namespace lamp
