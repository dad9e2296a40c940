// Weight repacking for the matrix-core 3x3x3 convolution kernels, one element per thread: shared by
// the per-call repack kernels and the batched one the network entry points use.
#pragma once
#include "internal.h"

namespace lamp {

// One thread moves one granule of 8 consecutive input channels (16 bytes) of the repacked layout.
// Forward: the granule is contiguous in W as well (one 16-byte load).  Data gradient: its 8 elements
// come from 8 rows of W; the threads are numbered with the output channel fastest, which is the
// contiguous dimension of W in that direction, so each of the 8 loads is coalesced across the wave.
__device__ __forceinline__ uint4 repack_gather8(const bf16_t* __restrict__ p, int64_t stride) {
    uint32_t r[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) r[e] = (uint32_t)p[(2 * e) * stride] | ((uint32_t)p[(2 * e + 1) * stride] << 16);
    return make_uint4(r[0], r[1], r[2], r[3]);
}

// Tiled kernel: the repacked weights are the kernel's LDS image,
//   wp[co block][chunk][group g][tap9 t9][plane][row][8],  oc = block*wrows + row, ic = chunk*16 + plane*8 + e,
// so that every 1 KB global -> LDS copy of the kernel reads consecutive memory (with [tap][oc][ic] a copy
// gathered 64 pieces of 16 bytes from 64 rows, and for many input channels those rows no longer stayed in
// L2).  Tap of (g, t9): kd = g, (kh, kw) = (t9/3, t9%3); bykh (8-deep tile, taps walked kh-major): kh = g,
// (kd, kw) = (t9/3, t9%3).  Values: forward W[oc][tap][ic], data gradient W[ic][26-tap][oc].
// 16 zero bytes behind the weights are the source of the zero padding.  g: granule index, Cin % 16 == 0.
__device__ __forceinline__ void repack_tile_gran(const bf16_t* __restrict__ w, bf16_t* __restrict__ wp, int64_t g, int Cout,
                                                 int Cin, int wrows, int dgrad, int bykh) {
    const int64_t total = (int64_t)27 * Cout * Cin;
    if (g == 0) *reinterpret_cast<uint4*>(wp + total) = make_uint4(0, 0, 0, 0);
    if (g >= total / 8) return;
    const int nchunks = Cin >> 4;
    int64_t r = g;
    const int row = (int)(r % wrows); r /= wrows;
    const int plane = (int)(r % 2); r /= 2;
    const int t9 = (int)(r % 9); r /= 9;
    const int grp = (int)(r % 3); r /= 3;
    const int chunk = (int)(r % nchunks);
    const int blk = (int)(r / nchunks);
    const int oc = blk * wrows + row, ic0 = chunk * 16 + plane * 8;
    const int t = bykh ? (t9 / 3) * 9 + grp * 3 + (t9 % 3) : grp * 9 + t9;
    uint4 v;
    if (!dgrad) v = *reinterpret_cast<const uint4*>(w + ((int64_t)oc * 27 + t) * Cin + ic0);
    else v = repack_gather8(w + ((int64_t)ic0 * 27 + (26 - t)) * Cout + oc, (int64_t)27 * Cout);
    *reinterpret_cast<uint4*>(wp + g * 8) = v;
}

}  // namespace lamp
