// Whole U-Net, one encoder partition, and sliding-window inference: host-side composition of the
// library's own entry points plus the window gather / Gaussian blend kernels.
//
// Data flow of a block  [conv -> InstanceNorm -> ReLU] x 2 : every conv writes its raw output z
// and the InstanceNorm statistics (conv epilogue); the activated tensor y is written once by the
// apply kernel.  The skip concat is never copied.  Where the matrix-core kernels apply (bf16, channel
// counts that are multiples of 32) it is not even materialised: the encoder output e_l and the
// up-sampled tensor are two contiguous tensors and the decoder's first conv reads its input
// channels from both (its data gradient writes to both), so that pooling, the transposed conv and
// their gradients never touch 64 of every 128 bytes.  Otherwise an encoder block's second conv
// writes straight into channels [0,C) of that level's concat buffer, where the transposed conv
// later writes channels [C,2C).  The backward recomputes the ReLU mask from z and the statistics.
#include <math.h>
#include <vector>
#include "internal.h"

namespace lamp {

struct ConvBuf {
    void* z; void* y; int ldy; float* stats;
    float* gate;   // squeeze-and-excitation variant: what the gate's forward leaves for its backward (second conv of a block)
};

struct Net {
    const lamp_unet_desc* u;
    int L, dt;
    size_t es;
    hipStream_t s;
    void* scratch; size_t scratch_bytes;
    void* gaux = nullptr;   // third gradient buffer (squeeze-and-excitation variant only)
    bool fwd_only = false;  // no backward follows: a block's first activated tensor feeds its second conv only
    int chan(int l) const { return u->base << (l - 1); }
    void dims(int l, int& d, int& h, int& w) const { d = u->d >> (l - 1); h = u->h >> (l - 1); w = u->w >> (l - 1); }
    int64_t vox(int l) const { int d, h, w; dims(l, d, h, w); return (int64_t)u->n * d * h * w; }
    lamp_tensor_desc td(int l, int c, int ldc) const {
        lamp_tensor_desc t; t.n = u->n; dims(l, t.d, t.h, t.w); t.c = c; t.ldc = ldc; t.dtype = dt; return t;
    }
};

static lamp_status unet_desc_ok(const lamp_unet_desc* u) {
    if (!u) return LAMP_ERR_NULL;
    if (u->levels < 1 || u->levels > 8 || u->base < 1 || u->in_ch < 1 || u->classes < 1 || u->classes > 16 || u->n < 1 ||
        u->d < 1 || u->h < 1 || u->w < 1)
        return LAMP_ERR_SHAPE;
    if (u->dtype != LAMP_F32 && u->dtype != LAMP_BF16) return LAMP_ERR_DTYPE;
    const int m = 1 << (u->levels - 1);
    if (u->d % m || u->h % m || u->w % m) return LAMP_ERR_SHAPE;
    if (!(u->eps >= 0.f)) return LAMP_ERR_SHAPE;
    if (u->se_ratio < 0 || u->se_ratio > 4096) return LAMP_ERR_SHAPE;
    return LAMP_OK;
}

static int per_conv(const lamp_unet_desc* u) { return u->affine ? 3 : 1; }
// parameter entries of one block: two convs and, in the squeeze-and-excitation variant, the gate's W1, b1, W2, b2
static int per_block(const lamp_unet_desc* u) { return 2 * per_conv(u) + (u->se_ratio ? 4 : 0); }
static int se_hidden(const lamp_unet_desc* u, int C) { const int r = C / u->se_ratio; return r < 1 ? 1 : r; }

// ---- scratch requirement: the largest per-call workspace of any layer ------------------------
static size_t block_scratch(const Net& nt, int l, int Cin, int Cout, bool bwd) {
    lamp_tensor_desc xi = nt.td(l, Cin, Cin), xo = nt.td(l, Cout, Cout);
    size_t m = lamp_conv3d_fwd_workspace_bytes(&xi, &xo, 1);
    size_t t = lamp_conv3d_fwd_workspace_bytes(&xo, &xo, 1);
    m = t > m ? t : m;
    if (bwd) {
        size_t c[] = {lamp_conv3d_wgrad_workspace_bytes(&xi, &xo), lamp_conv3d_wgrad_workspace_bytes(&xo, &xo),
                      lamp_conv3d_dgrad_workspace_bytes(&xo, &xi), lamp_conv3d_dgrad_workspace_bytes(&xo, &xo),
                      lamp_inorm_relu_bwd_workspace_bytes(&xo), lamp_conv3d_dgrad_inorm_relu_bwd_workspace_bytes(&xo, &xo)};
        for (size_t v : c) m = v > m ? v : m;
    }
    if (nt.u->se_ratio) {
        const size_t v = lamp_inorm_relu_se_workspace_bytes(&xo, se_hidden(nt.u, Cout));
        m = v > m ? v : m;
    }
    return m;
}

// last_apply == false leaves the second conv's output raw (z and its statistics): the consumer normalises
// while it loads.
static lamp_status block_fwd(Net& nt, int l, int Cin, int ldx, const void* x, int Cout, const void* const* P, int pi,
                             ConvBuf& c1, ConvBuf& c2, const void* x2 = nullptr, bool last_apply = true) {
    const lamp_unet_desc* u = nt.u;
    const int pc = per_conv(u);
    lamp_tensor_desc xd = nt.td(l, Cin, ldx), zd = nt.td(l, Cout, Cout);
    lamp_status st;
    if (x2) {   // input channels [0, Cin/2) in x, the rest in x2
        ConvParts parts{x2, Cin / 2, nullptr, 0, 0};
        st = mfma_conv_fwd(&xd, x, P[pi], false, &zd, c1.z, c1.stats, u->eps, nt.scratch, nt.scratch_bytes, nt.s, &parts);
    } else {
        st = lamp_conv3d_fwd(&xd, x, nullptr, P[pi], nullptr, &zd, c1.z, c1.stats, u->eps, nt.scratch, nt.scratch_bytes, nt.s);
    }
    if (st != LAMP_OK) return st;
    lamp_tensor_desc y1 = nt.td(l, Cout, c1.ldy);
    // Forward only, the first unit's activated tensor has one consumer, the second conv: where that conv takes the
    // matrix-core kernel it normalises the raw tensor while it loads it, and the tensor is never written.
    lamp_norm_in n1{c1.stats, u->affine ? (const float*)P[pi + 1] : nullptr, u->affine ? (const float*)P[pi + 2] : nullptr, Cout, 1};
    if (nt.fwd_only && !u->se_ratio && !tune("no_norm_on_load", 0) && mfma_conv_supported(&zd, &zd, &n1, nullptr)) {
        st = lamp_conv3d_fwd(&zd, c1.z, &n1, P[pi + pc], nullptr, &zd, c2.z, c2.stats, u->eps, nt.scratch, nt.scratch_bytes, nt.s);
    } else {
        st = lamp_inorm_relu(&zd, c1.z, n1.gamma, n1.beta, u->eps, &y1, c1.y, c1.stats, 1, nullptr, 0, nt.s);
        if (st != LAMP_OK) return st;
        st = lamp_conv3d_fwd(&y1, c1.y, nullptr, P[pi + pc], nullptr, &zd, c2.z, c2.stats, u->eps, nt.scratch,
                             nt.scratch_bytes, nt.s);
    }
    if (st != LAMP_OK) return st;
    lamp_tensor_desc y2 = nt.td(l, Cout, c2.ldy);
    if (u->se_ratio) {   // out = a1 + gate(mean a2) * a2: the gate on the second unit, the first unit's output as the shortcut
        const int ps = pi + 2 * pc;
        return lamp_inorm_relu_se(&zd, c2.z, c2.stats, u->affine ? (const float*)P[pi + pc + 1] : nullptr,
                                  u->affine ? (const float*)P[pi + pc + 2] : nullptr, se_hidden(u, Cout), (const float*)P[ps],
                                  (const float*)P[ps + 1], (const float*)P[ps + 2], (const float*)P[ps + 3], &y1, c1.y, &y2, c2.y,
                                  c2.gate, nt.scratch, nt.scratch_bytes, nt.s);
    }
    if (!last_apply) return st;
    return lamp_inorm_relu(&zd, c2.z, u->affine ? (const float*)P[pi + pc + 1] : nullptr,
                           u->affine ? (const float*)P[pi + pc + 2] : nullptr, u->eps, &y2, c2.y, c2.stats, 1, nullptr, 0,
                           nt.s);
}

// g: gradient w.r.t. c2.y, dense [.., Cout], overwritten.  gtmp: dense [.., Cout] scratch tensor.
// gx (nullable): receives the gradient w.r.t. the block input, channel stride ldgx.
static lamp_status block_bwd(Net& nt, int l, int Cin, int ldx, const void* x, int Cout, const void* const* P,
                             float* const* G, int pi, ConvBuf& c1, ConvBuf& c2, void* g, void* gtmp, void* gx, int ldgx,
                             float beta, const void* x2 = nullptr, void* gx2 = nullptr) {
    const lamp_unet_desc* u = nt.u;
    const int pc = per_conv(u);
    const bool af = u->affine != 0;
    lamp_tensor_desc zd = nt.td(l, Cout, Cout), xd = nt.td(l, Cin, ldx), y1 = nt.td(l, Cout, c1.ldy);
    lamp_status st;
    if (u->se_ratio) {
        // g reaches the first unit's output twice: through the gated second unit and, unchanged, through the shortcut.
        // dz2 goes to the third gradient buffer so that g survives until the two are added.
        const int ps = pi + 2 * pc;
        void* dz2 = nt.gaux;
        st = lamp_inorm_relu_se_bwd(&zd, g, &zd, c2.z, c2.stats, af ? (const float*)P[pi + pc + 1] : nullptr,
                                    af ? (const float*)P[pi + pc + 2] : nullptr, se_hidden(u, Cout), (const float*)P[ps],
                                    (const float*)P[ps + 2], c2.gate, &zd, dz2, af ? G[pi + pc + 1] : nullptr,
                                    af ? G[pi + pc + 2] : nullptr, G[ps], G[ps + 1], G[ps + 2], G[ps + 3], beta, nt.scratch,
                                    nt.scratch_bytes, nt.s);
        if (st != LAMP_OK) return st;
        st = lamp_conv3d_wgrad(&y1, c1.y, nullptr, &zd, dz2, G[pi + pc], nullptr, beta, nt.scratch, nt.scratch_bytes, nt.s);
        if (st != LAMP_OK) return st;
        st = lamp_conv3d_dgrad(&zd, dz2, P[pi + pc], &zd, gtmp, nt.scratch, nt.scratch_bytes, nt.s);
        if (st != LAMP_OK) return st;
        st = launch_add_inplace(gtmp, g, nvox(&zd) * Cout, nt.dt, nt.s);
        if (st != LAMP_OK) return st;
    } else {
        st = lamp_inorm_relu_bwd(&zd, g, &zd, c2.z, c2.stats, af ? (const float*)P[pi + pc + 1] : nullptr,
                                 af ? (const float*)P[pi + pc + 2] : nullptr, &zd, g, af ? G[pi + pc + 1] : nullptr,
                                 af ? G[pi + pc + 2] : nullptr, beta, nt.scratch, nt.scratch_bytes, nt.s);
        if (st != LAMP_OK) return st;
        st = lamp_conv3d_wgrad(&y1, c1.y, nullptr, &zd, g, G[pi + pc], nullptr, beta, nt.scratch, nt.scratch_bytes, nt.s);
        if (st != LAMP_OK) return st;
        // the data gradient of the second conv and the InstanceNorm + ReLU backward of the first as one call: the
        // sums of the latter come out of the former's epilogue
        st = lamp_conv3d_dgrad_inorm_relu_bwd(&zd, g, P[pi + pc], &zd, gtmp, &zd, c1.z, c1.stats,
                                              af ? (const float*)P[pi + 1] : nullptr, af ? (const float*)P[pi + 2] : nullptr,
                                              &zd, gtmp, af ? G[pi + 1] : nullptr, af ? G[pi + 2] : nullptr, beta, nt.scratch,
                                              nt.scratch_bytes, nt.s);
        if (st != LAMP_OK) return st;
    }
    if (u->se_ratio) {
        st = lamp_inorm_relu_bwd(&zd, gtmp, &zd, c1.z, c1.stats, af ? (const float*)P[pi + 1] : nullptr,
                                 af ? (const float*)P[pi + 2] : nullptr, &zd, gtmp, af ? G[pi + 1] : nullptr,
                                 af ? G[pi + 2] : nullptr, beta, nt.scratch, nt.scratch_bytes, nt.s);
        if (st != LAMP_OK) return st;
    }
    if (x2)   // two-part input (see block_fwd); the partial sums take the head of the scratch buffer
        st = mfma_wgrad(&xd, x, &zd, gtmp, G[pi], beta, nt.scratch, mfma_wgrad_ws_bytes(&xd, &zd), nt.s, x2, Cin / 2);
    else
        st = lamp_conv3d_wgrad(&xd, x, nullptr, &zd, gtmp, G[pi], nullptr, beta, nt.scratch, nt.scratch_bytes, nt.s);
    if (st != LAMP_OK) return st;
    if (gx) {
        lamp_tensor_desc gxd = nt.td(l, Cin, ldgx);
        if (gx2) {
            ConvParts parts{nullptr, 0, gx2, Cin / 2, ldgx};
            st = mfma_conv_fwd(&zd, gtmp, P[pi], true, &gxd, gx, nullptr, 0.f, nt.scratch, nt.scratch_bytes, nt.s, &parts);
        } else {
            st = lamp_conv3d_dgrad(&zd, gtmp, P[pi], &gxd, gx, nt.scratch, nt.scratch_bytes, nt.s);
        }
    }
    return st;
}

// ---- workspace layout -------------------------------------------------------------------------
struct Layout {
    // encoder level l (1-based index l-1), decoder level l (index l-1, l < L)
    std::vector<ConvBuf> e1, e2, d1, d2;
    // skip[l] = e_l's activated output, up[l] = the transposed conv's output, channel stride ldcat[l] (C when the
    // two are separate tensors, 2C when they are the halves of one concat buffer); gskip / gup: their gradients
    std::vector<void*> skip, up, gskip, gup, pooled;
    std::vector<int> ldcat;
    bool vcat;
    void *g0, *g1, *g2;
    void* scratch; size_t scratch_bytes;
    void* repack; size_t repack_bytes;   // repacked conv weights of the whole pass (one launch)
    size_t total;
};

static size_t repack_region_bytes(const Net& nt, int first, int last, bool whole, bool bwd);

// The concat stays virtual when every decoder block's first conv (2C -> C) takes the matrix-core
// kernels in all three directions.
static bool vcat_ok(const Net& nt) {
    if (tune("materialise_concat", 0) || nt.dt != LAMP_BF16 || nt.L < 2) return false;
    for (int l = 1; l < nt.L; ++l) {
        const int C = nt.chan(l);
        lamp_tensor_desc x2 = nt.td(l, 2 * C, C), z = nt.td(l, C, C);
        if (C % 32 || !mfma_conv_supported(&x2, &z, nullptr, nullptr) || !mfma_conv_supported(&z, &x2, nullptr, nullptr) ||
            !mfma_wgrad_supported(&x2, &z, nullptr))
            return false;
    }
    return true;
}

// Lays out every buffer of levels [first, last] of the encoder and (whole == true) the decoder.
// whole && first > 1 (the net's tail): the skips of levels below `first` and their gradients are the
// caller's tensors ext_skips[l-1] / ext_gskips[l-1]; this needs the virtual concat.
static void make_layout(Net& nt, int first, int last, bool whole, bool bwd, void* base, Layout& lay,
                        void* const* ext_skips, void* ext_pooled, void* const* ext_gskips = nullptr) {
    const lamp_unet_desc* u = nt.u;
    const int L = nt.L;
    Carver cv(base ? base : (void*)256, (size_t)1 << 62);
    auto take = [&](size_t b) -> void* { void* p = cv.take(b); return base ? p : nullptr; };
    lay.e1.assign(L, ConvBuf{}); lay.e2.assign(L, ConvBuf{}); lay.d1.assign(L, ConvBuf{}); lay.d2.assign(L, ConvBuf{});
    lay.skip.assign(L, nullptr); lay.up.assign(L, nullptr); lay.gskip.assign(L, nullptr); lay.gup.assign(L, nullptr);
    lay.pooled.assign(L, nullptr); lay.ldcat.assign(L, 0);
    lay.vcat = whole && vcat_ok(nt);
    const size_t es = nt.es;
    size_t scratch = 0, gmax = 0;
    if (whole)
        for (int l = 1; l < first; ++l) {
            const size_t tb = (size_t)nt.vox(l) * nt.chan(l) * es;
            lay.skip[l - 1] = ext_skips ? ext_skips[l - 1] : nullptr;
            lay.gskip[l - 1] = ext_gskips ? ext_gskips[l - 1] : nullptr;
            lay.up[l - 1] = take(tb);
            if (bwd) lay.gup[l - 1] = take(tb);
            lay.ldcat[l - 1] = nt.chan(l);
        }
    for (int l = first; l <= last; ++l) {
        const int C = nt.chan(l);
        const int Cin = l == 1 ? u->in_ch : nt.chan(l - 1);
        const size_t tb = (size_t)nt.vox(l) * C * es, sb = (size_t)u->n * C * 2 * sizeof(float);
        ConvBuf &a = lay.e1[l - 1], &b = lay.e2[l - 1];
        const bool se = u->se_ratio != 0;
        a.z = take(tb); a.stats = (float*)take(sb);
        a.y = bwd ? take(tb) : a.z; a.ldy = C;
        b.z = take(tb); b.stats = (float*)take(sb);
        if (se) b.gate = (float*)take((size_t)u->n * (4 * C + se_hidden(u, C)) * sizeof(float));
        if (whole && l < L) {
            if (lay.vcat) {
                lay.skip[l - 1] = take(tb); lay.up[l - 1] = take(tb); lay.ldcat[l - 1] = C;
                if (bwd) { lay.gskip[l - 1] = take(tb); lay.gup[l - 1] = take(tb); }
            } else {
                char* cat = (char*)take(2 * tb);
                lay.skip[l - 1] = cat; lay.up[l - 1] = base ? cat + (size_t)C * es : nullptr; lay.ldcat[l - 1] = 2 * C;
                if (bwd) {
                    char* gcat = (char*)take(2 * tb);
                    lay.gskip[l - 1] = gcat; lay.gup[l - 1] = base ? gcat + (size_t)C * es : nullptr;
                }
            }
            b.y = lay.skip[l - 1]; b.ldy = lay.ldcat[l - 1];
        } else if (!whole) {
            b.y = ext_skips ? ext_skips[l - first] : nullptr; b.ldy = C;
        } else {
            b.y = bwd || se ? take(tb) : b.z; b.ldy = C;
        }
        if (l < L) {
            const size_t pb = (size_t)nt.vox(l + 1) * C * es;
            if (!whole && l == last) lay.pooled[l - 1] = ext_pooled;
            else lay.pooled[l - 1] = take(pb);
        }
        size_t sc = block_scratch(nt, l, Cin, C, bwd);
        scratch = sc > scratch ? sc : scratch;
        gmax = tb > gmax ? tb : gmax;
    }
    if (whole) {
        for (int l = L - 1; l >= 1; --l) {
            const int C = nt.chan(l);
            const size_t tb = (size_t)nt.vox(l) * C * es, sb = (size_t)u->n * C * 2 * sizeof(float);
            ConvBuf &a = lay.d1[l - 1], &b = lay.d2[l - 1];
            a.z = take(tb); a.stats = (float*)take(sb); a.y = bwd ? take(tb) : a.z; a.ldy = C;
            b.z = take(tb); b.stats = (float*)take(sb); b.y = bwd || u->se_ratio ? take(tb) : b.z; b.ldy = C;
            if (u->se_ratio) b.gate = (float*)take((size_t)u->n * (4 * C + se_hidden(u, C)) * sizeof(float));
            size_t sc = block_scratch(nt, l, 2 * C, C, bwd);
            scratch = sc > scratch ? sc : scratch;
            gmax = tb > gmax ? tb : gmax;
            {
                lamp_tensor_desc xd = nt.td(l + 1, 2 * C, 2 * C), yd = nt.td(l, C, 2 * C);
                size_t t = lamp_convtr3d_workspace_bytes(&xd, &yd);
                scratch = t > scratch ? t : scratch;
                if (bwd) {
                    t = lamp_convtr3d_bwd_workspace_bytes(&xd, &yd);
                    scratch = t > scratch ? t : scratch;
                }
            }
        }
        if (bwd) {
            lamp_tensor_desc hd = nt.td(1, nt.chan(1), nt.chan(1));
            size_t t = lamp_head_ce_workspace_bytes(&hd, u->classes);
            scratch = t > scratch ? t : scratch;
        }
    }
    lay.g0 = lay.g1 = lay.g2 = nullptr;
    if (bwd) { lay.g0 = take(gmax); lay.g1 = take(gmax); if (u->se_ratio) lay.g2 = take(gmax); }
    lay.scratch_bytes = align_up(scratch);
    lay.scratch = take(lay.scratch_bytes);
    lay.repack_bytes = align_up(repack_region_bytes(nt, first, last, whole, bwd));
    lay.repack = lay.repack_bytes ? take(lay.repack_bytes) : nullptr;
    lay.total = align_up(cv.off) + 256;
}

static int enc_pi(const lamp_unet_desc* u, int l) { return (l - 1) * per_block(u); }
static int dec_pi(const lamp_unet_desc* u, int l) {  // index of "up Wt" of decoder level l
    return u->levels * per_block(u) + (u->levels - 1 - l) * (2 + per_block(u));
}
static int head_pi(const lamp_unet_desc* u) { return u->levels * per_block(u) + (u->levels - 1) * (2 + per_block(u)); }

// ---- conv weights repacked ahead of the pass, all in one launch ---------------------------------
// The 3x3x3 convs of levels [first, last] (and of the decoder when `whole`): parameter index, shapes.
struct ConvSpec { int pi, l, Cin, Cout; bool dgrad, parts; };
static void list_convs(const Net& nt, int first, int last, bool whole, int pbase, bool first_dgrad, std::vector<ConvSpec>& v) {
    const lamp_unet_desc* u = nt.u;
    const int pc = per_conv(u);
    for (int l = first; l <= last; ++l) {
        const int C = nt.chan(l), Cin = l == 1 ? u->in_ch : nt.chan(l - 1), pi = enc_pi(u, l) - pbase;
        v.push_back(ConvSpec{pi, l, Cin, C, l > first || first_dgrad, false});
        v.push_back(ConvSpec{pi + pc, l, C, C, true, false});
    }
    if (whole)
        for (int l = nt.L - 1; l >= 1; --l) {
            const int C = nt.chan(l), pi = dec_pi(u, l) + 2 - pbase;
            v.push_back(ConvSpec{pi, l, 2 * C, C, true, vcat_ok(nt)});
            v.push_back(ConvSpec{pi + pc, l, C, C, true, false});
        }
}
static size_t repack_region_bytes(const Net& nt, int first, int last, bool whole, bool bwd) {
    std::vector<ConvSpec> v;
    list_convs(nt, first, last, whole, 0, true, v);
    size_t b = 0;
    for (const ConvSpec& c : v) {
        lamp_tensor_desc xi = nt.td(c.l, c.Cin, c.Cin), xo = nt.td(c.l, c.Cout, c.Cout);
        if (conv_repack_kind(&xi, &xo, false) >= 0) b += conv_repack_bytes(&xi, &xo);
        if (bwd && conv_repack_kind(&xo, &xi, c.parts) >= 0) b += conv_repack_bytes(&xo, &xi);
    }
    return b;
}
// Fills the table and launches the repack of every conv weight the pass will use (fwd: forward
// layouts; dgrad: data-gradient layouts) into lay.repack.
static lamp_status prepare_repack(const Net& nt, const Layout& lay, int first, int last, bool whole, int pbase,
                                  const void* const* P, bool fwd, bool dgrad, bool first_dgrad, RepackTable& tab) {
    tab.n = 0;
    if (!lay.repack) return LAMP_OK;
    std::vector<ConvSpec> v;
    list_convs(nt, first, last, whole, pbase, first_dgrad, v);
    char* base = (char*)lay.repack;
    size_t off = 0;
    for (const ConvSpec& c : v) {
        lamp_tensor_desc xi = nt.td(c.l, c.Cin, c.Cin), xo = nt.td(c.l, c.Cout, c.Cout);
        for (int dir = 0; dir < 2; ++dir) {
            if (dir == 0 ? !fwd : !(dgrad && c.dgrad)) continue;
            const lamp_tensor_desc* xd = dir == 0 ? &xi : &xo;   // the conv's input / output in this direction
            const lamp_tensor_desc* zd = dir == 0 ? &xo : &xi;
            const int kind = conv_repack_kind(xd, zd, c.parts && dir == 1);
            if (kind < 0 || tab.n >= 64 || !aligned16(P[c.pi])) continue;
            const size_t b = conv_repack_bytes(xd, zd);
            if (off + b > lay.repack_bytes) continue;
            tab.e[tab.n++] = RepackJob{P[c.pi], base + off, zd->c, xd->c, dir, kind};
            off += b;
        }
    }
    return launch_repack_batch(tab.e, tab.n, nt.s);
}
struct RepackScope {   // the calling thread's conv calls see the table for the duration of the pass
    explicit RepackScope(const RepackTable* t) { set_repack_table(t); }
    ~RepackScope() { set_repack_table(nullptr); }
};

static lamp_status encoder_fwd(Net& nt, Layout& lay, int first, int last, const void* const* P, int pbase, const void* x) {
    const lamp_unet_desc* u = nt.u;
    const void* cur = x;
    int cur_c = first == 1 ? u->in_ch : nt.chan(first - 1);
    for (int l = first; l <= last; ++l) {
        const int C = nt.chan(l);
        // Above the bottom level the block's second InstanceNorm + ReLU is applied by the pooling pass, which
        // writes the activated tensor (the skip) and its pooled version from one read of the raw conv output.
        const bool pooled = l < nt.L;
        const int pi = enc_pi(u, l) - pbase;
        lamp_status st = block_fwd(nt, l, cur_c, cur_c, cur, C, P, pi, lay.e1[l - 1], lay.e2[l - 1], nullptr, !pooled);
        if (st != LAMP_OK) return st;
        if (pooled && u->se_ratio) {   // the gate's pass has written the block's output: a plain pooling pass follows
            lamp_tensor_desc yd2 = nt.td(l, C, lay.e2[l - 1].ldy), pd = nt.td(l + 1, C, C);
            st = lamp_maxpool2_fwd(&yd2, lay.e2[l - 1].y, nullptr, &pd, lay.pooled[l - 1], nt.s);
            if (st != LAMP_OK) return st;
            cur = lay.pooled[l - 1];
        } else if (pooled) {
            const int pc = per_conv(u);
            lamp_norm_in zn{lay.e2[l - 1].stats, u->affine ? (const float*)P[pi + pc + 1] : nullptr,
                            u->affine ? (const float*)P[pi + pc + 2] : nullptr, C, 1};
            lamp_tensor_desc zd = nt.td(l, C, C), yd = nt.td(l + 1, C, C);
            st = inorm_relu_maxpool2(&zd, lay.e2[l - 1].z, &zn, lay.e2[l - 1].y, lay.e2[l - 1].ldy, &yd, lay.pooled[l - 1], nt.s);
            if (st != LAMP_OK) return st;
            cur = lay.pooled[l - 1];
        }
        cur_c = C;
    }
    return LAMP_OK;
}

// g_init: gradient w.r.t. the pooled output of level `last` (any buffer, read only), or, when
// last == L, w.r.t. e_L's activated output, in which case it must be lay.g0 (it is overwritten).
// skip_g[l-1] / ldsg[l-1]: gradient arriving through the skip copy of e_l (levels below L).
// dx_out (nullable): receives the gradient w.r.t. the partition's input.
static lamp_status encoder_bwd(Net& nt, Layout& lay, int first, int last, const void* const* P, float* const* G,
                               int pbase, const void* x, const void* g_init, const void* const* skip_g, const int* ldsg,
                               void* dx_out, float beta) {
    const lamp_unet_desc* u = nt.u;
    const void* gin = g_init;
    void* bufA = lay.g0;
    void* bufB = lay.g1;
    for (int l = last; l >= first; --l) {
        const int C = nt.chan(l);
        void *g, *other;
        if (l < nt.L) {
            lamp_tensor_desc xd = nt.td(l, C, lay.e2[l - 1].ldy), gd = nt.td(l + 1, C, C), ad = nt.td(l, C, ldsg[l - 1]),
                             od = nt.td(l, C, C);
            lamp_status st = lamp_maxpool2_bwd(&xd, lay.e2[l - 1].y, nullptr, &gd, gin, &ad, skip_g[l - 1], &od, bufA, nt.s);
            if (st != LAMP_OK) return st;
            g = bufA; other = bufB;
        } else {
            g = lay.g0; other = lay.g1;
        }
        const int Cin = l == 1 ? u->in_ch : nt.chan(l - 1);
        const void* xin = l == first ? x : lay.pooled[l - 2];
        // the input gradient may reuse g: g is dead once the first conv's dz sits in `other`
        void* dst = l > first ? g : dx_out;
        lamp_status st = block_bwd(nt, l, Cin, Cin, xin, C, P, G, enc_pi(u, l) - pbase, lay.e1[l - 1], lay.e2[l - 1], g,
                                   other, dst, Cin, beta);
        if (st != LAMP_OK) return st;
        gin = g;
        bufA = other; bufB = g;
    }
    return LAMP_OK;
}

}  // namespace lamp

using namespace lamp;

extern "C" int32_t lamp_unet_param_count(const lamp_unet_desc* u) {
    if (unet_desc_ok(u) != LAMP_OK) return 0;
    return head_pi(u) + 2;
}

extern "C" int64_t lamp_unet_param_numel(const lamp_unet_desc* u, int32_t idx) {
    if (unet_desc_ok(u) != LAMP_OK || idx < 0 || idx >= lamp_unet_param_count(u)) return 0;
    const int pc = per_conv(u), pb = per_block(u), L = u->levels;
    auto ch = [&](int l) { return (int64_t)u->base << (l - 1); };
    auto conv_entry = [&](int64_t Cin, int64_t Cout, int k) -> int64_t {  // k: position inside a block
        if (k >= 2 * pc) {   // the gate: W1 [cr][C], b1 [cr], W2 [C][cr], b2 [C]
            const int64_t cr = se_hidden(u, (int)Cout);
            const int64_t n[4] = {cr * Cout, cr, Cout * cr, Cout};
            return n[k - 2 * pc];
        }
        int which = k / pc, sub = k % pc;
        if (sub) return Cout;
        return Cout * 27 * (which == 0 ? Cin : Cout);
    };
    if (idx < L * pb) {
        int l = idx / pb + 1;
        return conv_entry(l == 1 ? u->in_ch : ch(l - 1), ch(l), idx % pb);
    }
    idx -= L * pb;
    const int per = 2 + pb;
    if (idx < (L - 1) * per) {
        int l = L - 1 - idx / per, k = idx % per;
        if (k == 0) return ch(l + 1) * 8 * ch(l);
        if (k == 1) return ch(l);
        return conv_entry(2 * ch(l), ch(l), k - 2);
    }
    idx -= (L - 1) * per;
    return idx == 0 ? (int64_t)u->classes * ch(1) : u->classes;
}

extern "C" size_t lamp_unet_workspace_bytes(const lamp_unet_desc* u, int with_backward) {
    if (unet_desc_ok(u) != LAMP_OK) return 0;
    Net nt{u, u->levels, u->dtype, esize(u->dtype), nullptr, nullptr, 0};
    Layout lay;
    make_layout(nt, 1, u->levels, true, with_backward != 0, nullptr, lay, nullptr, nullptr);
    return lay.total;
}

// The net's tail: encoder blocks first..L, the whole decoder and the head, fed with the pooled output
// of block first-1 and the skips e_1..e_{first-1} (Eq. 3: the copies e_{l,1} that travel past the cut).
// phase 0: the whole pass; 1: the forward up to the head's input, laid out for a backward;
// 2: head, loss and the backward over what phase 1 left in the workspace.
struct TailIO {
    int first;
    const void* const* skips;   // [first-1]
    void* const* d_skips;       // [first-1], written (backward)
    void* d_x;                  // gradient w.r.t. the tail's input (backward), nullable
    int phase;
    int64_t norm_count;         // voxel count of the loss mean (0: this call's own)
    float loss_beta;
};

static lamp_status unet_run(const lamp_unet_desc* u, const void* const* P, const void* x, const int32_t* labels,
                            float* logits, float* loss, float* const* G, float beta, bool bwd, void* ws, size_t ws_bytes,
                            void* stream, const TailIO* tail = nullptr) {
    lamp_status st = unet_desc_ok(u);
    if (st != LAMP_OK) return st;
    if (!P || !x) return LAMP_ERR_NULL;
    const int first = tail ? tail->first : 1, phase = tail ? tail->phase : 0;
    if (first < 1 || first > u->levels) return LAMP_ERR_SHAPE;
    const int pbase = enc_pi(u, first);
    const int np = lamp_unet_param_count(u) - pbase;
    for (int i = 0; i < np; ++i)
        if (!P[i]) return LAMP_ERR_NULL;
    if (bwd) {
        if (!labels || !loss || !G) return LAMP_ERR_NULL;
        for (int i = 0; i < np; ++i)
            if (!G[i]) return LAMP_ERR_NULL;
        if (beta != 0.f && beta != 1.f) return LAMP_ERR_SHAPE;
    } else if (!logits) return LAMP_ERR_NULL;
    if (first > 1) {
        if (!tail->skips || (bwd && !tail->d_skips)) return LAMP_ERR_NULL;
        for (int l = 1; l < first; ++l) {
            if (!tail->skips[l - 1] || (bwd && !tail->d_skips[l - 1])) return LAMP_ERR_NULL;
            if (!aligned16(tail->skips[l - 1]) || (bwd && !aligned16(tail->d_skips[l - 1]))) return LAMP_ERR_ALIGN;
        }
        if (tail->d_x && !aligned16(tail->d_x)) return LAMP_ERR_ALIGN;
    }
    if (!aligned16(x) || !aligned16(ws)) return LAMP_ERR_ALIGN;
    Net nt{u, u->levels, u->dtype, esize(u->dtype), (hipStream_t)stream, nullptr, 0};
    const int L = nt.L;
    if (first > 1 && !vcat_ok(nt)) return LAMP_ERR_UNSUPPORTED;   // external skips need the two-tensor concat
    Layout lay;
    make_layout(nt, first, L, true, bwd, nullptr, lay, nullptr, nullptr);
    if (!ws || ws_bytes < lay.total) return LAMP_ERR_WORKSPACE;
    make_layout(nt, first, L, true, bwd, ws, lay, tail ? (void* const*)tail->skips : nullptr, nullptr,
                tail && bwd ? tail->d_skips : nullptr);
    nt.scratch = lay.scratch; nt.scratch_bytes = lay.scratch_bytes;
    nt.gaux = lay.g2;
    nt.fwd_only = !bwd;
    const bool first_dgrad = tail && tail->d_x;
    RepackTable tab;
    if ((st = prepare_repack(nt, lay, first, L, true, pbase, P, phase != 2, bwd && phase != 1, first_dgrad, tab)) != LAMP_OK)
        return st;
    RepackScope scope(&tab);

    const int C1 = nt.chan(1), hp = head_pi(u) - pbase;
    lamp_tensor_desc hd = nt.td(1, C1, C1);
    const void* top = L > 1 ? lay.d2[0].y : lay.e2[0].y;
    hd.ldc = L > 1 ? lay.d2[0].ldy : lay.e2[0].ldy;
    // the matrix-core head normalises on load only where its 32-voxel groups stay inside one sample
    const bool head_norm = ((int64_t)u->d * u->h * u->w) % 32 == 0 && !u->se_ratio;
    if (phase != 2) {
        if ((st = encoder_fwd(nt, lay, first, L, P, pbase, x)) != LAMP_OK) return st;
        const void* cur = lay.e2[L - 1].y;
        for (int l = L - 1; l >= 1; --l) {
            const int C = nt.chan(l), pi = dec_pi(u, l) - pbase;
            const int ldc = lay.ldcat[l - 1];
            lamp_tensor_desc xd = nt.td(l + 1, 2 * C, 2 * C), yd = nt.td(l, C, ldc);
            st = lamp_convtr3d(&xd, cur, nullptr, P[pi], (const float*)P[pi + 1], &yd, lay.up[l - 1], nt.scratch,
                               nt.scratch_bytes, nt.s);
            if (st != LAMP_OK) return st;
            // inference: the last block's output feeds only the head, which normalises while it loads
            st = block_fwd(nt, l, 2 * C, ldc, lay.skip[l - 1], C, P, pi + 2, lay.d1[l - 1], lay.d2[l - 1],
                           lay.vcat ? lay.up[l - 1] : nullptr, bwd || l > 1 || !head_norm);
            if (st != LAMP_OK) return st;
            cur = lay.d2[l - 1].y;
        }
        if (!bwd && L > 1 && head_norm) {
            const int pc = per_conv(u), pi2 = dec_pi(u, 1) - pbase + 2 + pc;   // the last block's second conv
            lamp_norm_in hn{lay.d2[0].stats, u->affine ? (const float*)P[pi2 + 1] : nullptr,
                            u->affine ? (const float*)P[pi2 + 2] : nullptr, C1, 1};
            lamp_tensor_desc zd = nt.td(1, C1, C1);
            return lamp_head_fwd(&zd, lay.d2[0].z, &hn, P[hp], (const float*)P[hp + 1], u->classes, logits, nt.s);
        }
        if (!bwd) return lamp_head_fwd(&hd, top, nullptr, P[hp], (const float*)P[hp + 1], u->classes, logits, nt.s);
        if (phase == 1) return LAMP_OK;
    }

    // ---- backward ----
    lamp_tensor_desc gd = nt.td(1, C1, C1);
    st = head_ce_run(&hd, top, nullptr, P[hp], (const float*)P[hp + 1], u->classes, labels, logits, loss, &gd, lay.g0, G[hp],
                     G[hp + 1], beta, tail ? tail->norm_count : 0, tail ? tail->loss_beta : 0.f, nt.scratch, nt.scratch_bytes,
                     nt.s);
    if (st != LAMP_OK) return st;
    std::vector<const void*> skip_g(L, nullptr);
    std::vector<int> ldsg(L, 0);
    for (int l = 1; l <= L - 1; ++l) {
        const int C = nt.chan(l), pi = dec_pi(u, l) - pbase;
        const int ldc = lay.ldcat[l - 1];
        st = block_bwd(nt, l, 2 * C, ldc, lay.skip[l - 1], C, P, G, pi + 2, lay.d1[l - 1], lay.d2[l - 1], lay.g0, lay.g1,
                       lay.gskip[l - 1], ldc, beta, lay.vcat ? lay.up[l - 1] : nullptr, lay.vcat ? lay.gup[l - 1] : nullptr);
        if (st != LAMP_OK) return st;
        skip_g[l - 1] = lay.gskip[l - 1];
        ldsg[l - 1] = ldc;
        lamp_tensor_desc xd = nt.td(l + 1, 2 * C, 2 * C), dyd = nt.td(l, C, ldc), dxd = nt.td(l + 1, 2 * C, 2 * C);
        const void* xin = l + 1 == L ? lay.e2[L - 1].y : lay.d2[l].y;
        xd.ldc = l + 1 == L ? lay.e2[L - 1].ldy : lay.d2[l].ldy;
        st = lamp_convtr3d_bwd(&xd, xin, nullptr, P[pi], &dyd, lay.gup[l - 1], &dxd, lay.g0, G[pi], G[pi + 1], beta, nt.scratch,
                               nt.scratch_bytes, nt.s);
        if (st != LAMP_OK) return st;
    }
    return encoder_bwd(nt, lay, first, L, P, G, pbase, x, lay.g0, skip_g.data(), ldsg.data(), tail ? tail->d_x : nullptr, beta);
}

extern "C" lamp_status lamp_unet_fwd(const lamp_unet_desc* u, const void* const* params, const void* x, float* logits,
                                     void* ws, size_t ws_bytes, void* stream) {
    return unet_run(u, params, x, nullptr, logits, nullptr, nullptr, 0.f, false, ws, ws_bytes, stream);
}

extern "C" lamp_status lamp_unet_fwd_bwd(const lamp_unet_desc* u, const void* const* params, const void* x,
                                         const int32_t* labels, float* logits, float* loss, float* const* grads, float beta,
                                         void* ws, size_t ws_bytes, void* stream) {
    return unet_run(u, params, x, labels, logits, loss, grads, beta, true, ws, ws_bytes, stream);
}

// ---- one encoder partition --------------------------------------------------------------------
static lamp_status stage_ok(const lamp_unet_desc* u, int first, int last) {
    lamp_status st = unet_desc_ok(u);
    if (st != LAMP_OK) return st;
    if (u->se_ratio) return LAMP_ERR_UNSUPPORTED;   // the partition entry points serve the plain U-Net
    if (first < 1 || last < first || last >= u->levels) return LAMP_ERR_SHAPE;
    return LAMP_OK;
}

// The stage works on a descriptor whose level numbering is the whole net's but whose d,h,w are the
// partition's input dims: shift them so that level `first` has those dims.
static lamp_unet_desc stage_desc(const lamp_unet_desc* u, int first) {
    lamp_unet_desc v = *u;
    v.d = u->d << (first - 1); v.h = u->h << (first - 1); v.w = u->w << (first - 1);
    return v;
}

extern "C" size_t lamp_unet_stage_workspace_bytes(const lamp_unet_desc* u, int first, int last, int with_backward) {
    if (stage_ok(u, first, last) != LAMP_OK) return 0;
    const int m = 1 << (last - first + 1);
    if (u->d % m || u->h % m || u->w % m) return 0;
    lamp_unet_desc v = stage_desc(u, first);
    Net nt{&v, v.levels, v.dtype, esize(v.dtype), nullptr, nullptr, 0};
    Layout lay;
    make_layout(nt, first, last, false, with_backward != 0, nullptr, lay, nullptr, nullptr);
    return lay.total;
}

extern "C" lamp_status lamp_unet_stage_fwd(const lamp_unet_desc* u, int first, int last, const void* const* params,
                                           const void* x, void* pooled, void* const* skips, void* ws, size_t ws_bytes,
                                           void* stream) {
    lamp_status st = stage_ok(u, first, last);
    if (st != LAMP_OK) return st;
    const int m = 1 << (last - first + 1);
    if (u->d % m || u->h % m || u->w % m) return LAMP_ERR_SHAPE;
    if (!params || !x || !pooled || !skips) return LAMP_ERR_NULL;
    for (int i = 0; i <= last - first; ++i)
        if (!skips[i]) return LAMP_ERR_NULL;
    for (int i = 0; i < (last - first + 1) * 2 * per_conv(u); ++i)
        if (!params[i]) return LAMP_ERR_NULL;
    if (!aligned16(x) || !aligned16(ws) || !aligned16(pooled)) return LAMP_ERR_ALIGN;
    // the backward needs what the forward leaves behind, so the forward always lays out for it
    if (!ws || ws_bytes < lamp_unet_stage_workspace_bytes(u, first, last, 1)) return LAMP_ERR_WORKSPACE;
    lamp_unet_desc v = stage_desc(u, first);
    Net nt{&v, v.levels, v.dtype, esize(v.dtype), (hipStream_t)stream, nullptr, 0};
    Layout lay;
    make_layout(nt, first, last, false, true, ws, lay, skips, pooled);
    nt.scratch = lay.scratch; nt.scratch_bytes = lay.scratch_bytes;
    RepackTable tab;
    if ((st = prepare_repack(nt, lay, first, last, false, enc_pi(&v, first), params, true, false, false, tab)) != LAMP_OK) return st;
    RepackScope scope(&tab);
    return encoder_fwd(nt, lay, first, last, params, enc_pi(&v, first), x);
}

extern "C" lamp_status lamp_unet_stage_bwd(const lamp_unet_desc* u, int first, int last, const void* const* params,
                                           const void* x, const void* const* skips, const void* d_pooled,
                                           const void* const* d_skips, float* const* grads, float beta, void* dx, void* ws,
                                           size_t ws_bytes, void* stream) {
    lamp_status st = stage_ok(u, first, last);
    if (st != LAMP_OK) return st;
    const int m = 1 << (last - first + 1);
    if (u->d % m || u->h % m || u->w % m) return LAMP_ERR_SHAPE;
    if (!params || !x || !skips || !d_pooled || !d_skips || !grads) return LAMP_ERR_NULL;
    for (int i = 0; i <= last - first; ++i)
        if (!skips[i] || !d_skips[i]) return LAMP_ERR_NULL;
    for (int i = 0; i < (last - first + 1) * 2 * per_conv(u); ++i)
        if (!params[i] || !grads[i]) return LAMP_ERR_NULL;
    if (beta != 0.f && beta != 1.f) return LAMP_ERR_SHAPE;
    if (dx && first == 1) return LAMP_ERR_UNSUPPORTED;  // the first block's input is data
    if (!aligned16(x) || !aligned16(ws) || !aligned16(d_pooled)) return LAMP_ERR_ALIGN;
    if (!ws || ws_bytes < lamp_unet_stage_workspace_bytes(u, first, last, 1)) return LAMP_ERR_WORKSPACE;
    lamp_unet_desc v = stage_desc(u, first);
    Net nt{&v, v.levels, v.dtype, esize(v.dtype), (hipStream_t)stream, nullptr, 0};
    Layout lay;
    make_layout(nt, first, last, false, true, ws, lay, (void* const*)skips, nullptr);
    nt.scratch = lay.scratch; nt.scratch_bytes = lay.scratch_bytes;
    RepackTable tab;
    if ((st = prepare_repack(nt, lay, first, last, false, enc_pi(&v, first), params, false, true, dx != nullptr, tab)) != LAMP_OK)
        return st;
    RepackScope scope(&tab);
    std::vector<const void*> sg(v.levels, nullptr);
    std::vector<int> ld(v.levels, 0);
    for (int l = first; l <= last; ++l) { sg[l - 1] = d_skips[l - first]; ld[l - 1] = nt.chan(l); }
    return encoder_bwd(nt, lay, first, last, params, grads, enc_pi(&v, first), x, d_pooled, sg.data(), ld.data(), dx, beta);
}

// ---- the net's tail (second pipeline partition) and the two-partition micro-batch schedule -----------
static lamp_status tail_ok(const lamp_unet_desc* u, int first) {
    lamp_status st = unet_desc_ok(u);
    if (st != LAMP_OK) return st;
    if (u->se_ratio) return LAMP_ERR_UNSUPPORTED;
    if (first < 2 || first > u->levels) return LAMP_ERR_SHAPE;
    return LAMP_OK;
}

extern "C" int32_t lamp_unet_tail_param_offset(const lamp_unet_desc* u, int32_t first) {
    if (tail_ok(u, first) != LAMP_OK) return -1;
    return enc_pi(u, first);
}

extern "C" size_t lamp_unet_tail_workspace_bytes(const lamp_unet_desc* u, int first, int with_backward) {
    if (tail_ok(u, first) != LAMP_OK) return 0;
    Net nt{u, u->levels, u->dtype, esize(u->dtype), nullptr, nullptr, 0};
    if (!vcat_ok(nt)) return 0;
    Layout lay;
    make_layout(nt, first, u->levels, true, with_backward != 0, nullptr, lay, nullptr, nullptr);
    return lay.total;
}

extern "C" lamp_status lamp_unet_tail_fwd(const lamp_unet_desc* u, int first, const void* const* params, const void* x,
                                          const void* const* skips, float* logits, void* ws, size_t ws_bytes, void* stream) {
    lamp_status st = tail_ok(u, first);
    if (st != LAMP_OK) return st;
    TailIO io{first, skips, nullptr, nullptr, 0, 0, 0.f};
    return unet_run(u, params, x, nullptr, logits, nullptr, nullptr, 0.f, false, ws, ws_bytes, stream, &io);
}

extern "C" lamp_status lamp_unet_tail_fwd_bwd(const lamp_unet_desc* u, int first, const void* const* params, const void* x,
                                              const void* const* skips, const int32_t* labels, float* logits, float* loss,
                                              float* const* grads, float beta, void* d_x, void* const* d_skips, void* ws,
                                              size_t ws_bytes, void* stream) {
    lamp_status st = tail_ok(u, first);
    if (st != LAMP_OK) return st;
    TailIO io{first, skips, d_skips, d_x, 0, 0, 0.f};
    return unet_run(u, params, x, labels, logits, loss, grads, beta, true, ws, ws_bytes, stream, &io);
}

namespace lamp {

// Per-micro-batch buffers of the two-partition schedule, carved from the caller's workspace.
struct PipeSlot {
    void* stage_ws; void* tail_ws;
    void* pooled; void* d_pooled;
    void* skips[8]; void* d_skips[8];
};
struct PipeLayout {
    size_t stage_bytes, tail_bytes, total;
    std::vector<PipeSlot> slot;
};

static bool pipe_layout(const lamp_unet_desc* u, int cut, int M, void* base, PipeLayout& pl) {
    Net nt{u, u->levels, u->dtype, esize(u->dtype), nullptr, nullptr, 0};
    pl.stage_bytes = lamp_unet_stage_workspace_bytes(u, 1, cut, 1);
    pl.tail_bytes = lamp_unet_tail_workspace_bytes(u, cut + 1, 1);
    if (!pl.stage_bytes || !pl.tail_bytes) return false;
    Carver cv(base ? base : (void*)256, (size_t)1 << 62);
    auto take = [&](size_t b) -> void* { void* p = cv.take(b); return base ? p : nullptr; };
    pl.slot.assign(M, PipeSlot{});
    for (int m = 0; m < M; ++m) {
        PipeSlot& sl = pl.slot[m];
        sl.stage_ws = take(pl.stage_bytes);
        sl.tail_ws = take(pl.tail_bytes);
        const size_t pb = (size_t)nt.vox(cut + 1) * nt.chan(cut) * nt.es;
        sl.pooled = take(pb); sl.d_pooled = take(pb);
        for (int l = 1; l <= cut; ++l) {
            const size_t tb = (size_t)nt.vox(l) * nt.chan(l) * nt.es;
            sl.skips[l - 1] = take(tb); sl.d_skips[l - 1] = take(tb);
        }
    }
    pl.total = align_up(cv.off) + 256;
    return true;
}

}  // namespace lamp

static lamp_status pipe_ok(const lamp_unet_desc* u, int cut, int M) {
    lamp_status st = unet_desc_ok(u);
    if (st != LAMP_OK) return st;
    if (u->se_ratio) return LAMP_ERR_UNSUPPORTED;
    if (cut < 1 || cut >= u->levels || M < 1 || M > 64) return LAMP_ERR_SHAPE;
    return LAMP_OK;
}

extern "C" size_t lamp_unet_pipeline_workspace_bytes(const lamp_unet_desc* u, int cut, int micro_batches) {
    if (pipe_ok(u, cut, micro_batches) != LAMP_OK) return 0;
    PipeLayout pl;
    return pipe_layout(u, cut, micro_batches, nullptr, pl) ? pl.total : 0;
}

#define LAMP_PIPE_HIP(call)                         \
    do {                                            \
        if (st == LAMP_OK && (call) != hipSuccess) st = LAMP_ERR_HIP; \
    } while (0)

extern "C" lamp_status lamp_unet_pipeline_fwd_bwd(const lamp_unet_desc* u, int cut, int micro_batches,
                                                  const void* const* params, const void* x, const int32_t* labels,
                                                  float* logits, float* loss, float* const* grads, float beta, void* ws,
                                                  size_t ws_bytes, void* stream, void* aux_stream) {
    lamp_status st = pipe_ok(u, cut, micro_batches);
    if (st != LAMP_OK) return st;
    const int M = micro_batches, L = u->levels;
    if (!params || !x || !labels || !loss || !grads) return LAMP_ERR_NULL;
    const int np = lamp_unet_param_count(u);
    for (int i = 0; i < np; ++i)
        if (!params[i] || !grads[i]) return LAMP_ERR_NULL;
    if (beta != 0.f && beta != 1.f) return LAMP_ERR_SHAPE;
    if (stream == aux_stream) return LAMP_ERR_SHAPE;   // the two partitions run on two different streams
    if (!aligned16(x) || !aligned16(ws)) return LAMP_ERR_ALIGN;
    PipeLayout pl;
    if (!pipe_layout(u, cut, M, nullptr, pl)) return LAMP_ERR_UNSUPPORTED;
    if (!ws || ws_bytes < pl.total) return LAMP_ERR_WORKSPACE;
    pipe_layout(u, cut, M, ws, pl);
    Net nt{u, L, u->dtype, esize(u->dtype), nullptr, nullptr, 0};
    const size_t x_mb = (size_t)nt.vox(1) * u->in_ch * nt.es;   // bytes of one micro-batch of x
    if (x_mb % 16) return LAMP_ERR_ALIGN;
    const int64_t v_mb = nt.vox(1);
    const int toff = enc_pi(u, cut + 1);
    hipStream_t s0 = (hipStream_t)stream, s1 = (hipStream_t)aux_stream;

    // events: [0, M) forward of partition 0 done, [M, 2M) backward of partition 1 done, 2M fork, 2M+1 join
    std::vector<hipEvent_t> ev(2 * M + 2, nullptr);
    for (size_t i = 0; i < ev.size(); ++i)
        if (hipEventCreateWithFlags(&ev[i], hipEventDisableTiming) != hipSuccess) {
            for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(ev[j]);
            return LAMP_ERR_HIP;
        }
    LAMP_PIPE_HIP(hipEventRecord(ev[2 * M], s0));
    LAMP_PIPE_HIP(hipStreamWaitEvent(s1, ev[2 * M], 0));
    auto xm = [&](int m) { return (const char*)x + (size_t)m * x_mb; };
    auto tail_io = [&](int m, int phase, bool first_bwd) {
        const PipeSlot& sl = pl.slot[m];
        return TailIO{cut + 1, (const void* const*)sl.skips, (void* const*)sl.d_skips, sl.d_pooled, phase,
                      (int64_t)M * v_mb, first_bwd ? 0.f : 1.f};
    };
    // forward: at clock t partition 0 runs micro-batch t and partition 1 micro-batch t-1
    for (int t = 0; t <= M && st == LAMP_OK; ++t) {
        if (t < M) {
            const PipeSlot& sl = pl.slot[t];
            st = lamp_unet_stage_fwd(u, 1, cut, params, xm(t), sl.pooled, (void* const*)sl.skips, sl.stage_ws, pl.stage_bytes,
                                     s0);
            LAMP_PIPE_HIP(hipEventRecord(ev[t], s0));
        }
        if (t >= 1 && st == LAMP_OK) {
            const int m = t - 1;
            const PipeSlot& sl = pl.slot[m];
            LAMP_PIPE_HIP(hipStreamWaitEvent(s1, ev[m], 0));
            TailIO io = tail_io(m, 1, false);
            if (st == LAMP_OK)
                st = unet_run(u, params + toff, sl.pooled, labels + (size_t)m * v_mb, nullptr, loss, grads + toff, beta, true,
                              sl.tail_ws, pl.tail_bytes, s1, &io);
        }
    }
    // backward, micro-batches in reverse: partition 1 first, partition 0 one clock behind it
    for (int t = 0; t < M && st == LAMP_OK; ++t) {
        const int m = M - 1 - t;
        const PipeSlot& sl = pl.slot[m];
        const float b = t == 0 ? beta : 1.f;
        TailIO io = tail_io(m, 2, t == 0);
        st = unet_run(u, params + toff, sl.pooled, labels + (size_t)m * v_mb,
                      logits ? logits + (size_t)m * v_mb * u->classes : nullptr, loss, grads + toff, b, true, sl.tail_ws,
                      pl.tail_bytes, s1, &io);
        LAMP_PIPE_HIP(hipEventRecord(ev[M + m], s1));
        LAMP_PIPE_HIP(hipStreamWaitEvent(s0, ev[M + m], 0));
        if (st == LAMP_OK)
            st = lamp_unet_stage_bwd(u, 1, cut, params, xm(m), (const void* const*)sl.skips, sl.d_pooled,
                                     (const void* const*)sl.d_skips, grads, b, nullptr, sl.stage_ws, pl.stage_bytes, s0);
    }
    // join: whatever was enqueued on the second stream completes before later work on `stream`
    if (hipEventRecord(ev[2 * M + 1], s1) != hipSuccess || hipStreamWaitEvent(s0, ev[2 * M + 1], 0) != hipSuccess)
        if (st == LAMP_OK) st = LAMP_ERR_HIP;
    for (hipEvent_t e : ev) (void)hipEventDestroy(e);
    return st;
}

// ---- sliding-window inference -------------------------------------------------------------------
namespace lamp {

static int sw_stride(int patch, float overlap) { return (int)lroundf(patch * (1.0f - overlap)); }
static int sw_count1(int len, int patch, int stride) { return len <= patch ? 1 : (len - patch + stride - 1) / stride + 1; }

template <typename T>
__global__ __launch_bounds__(256) void sw_gather_kernel(const T* __restrict__ vol, T* __restrict__ win, int D, int H, int W,
                                                        int C, int P, int stride, int cd, int ch, int cw) {
    const int64_t per = (int64_t)P * P * P * C;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= per * cd * ch * cw) return;
    const int wi = (int)(idx / per);
    int64_t r = idx % per;
    const int c = (int)(r % C); r /= C;
    const int k = (int)(r % P); r /= P;
    const int j = (int)(r % P);
    const int i = (int)(r / P);
    const int iw = wi % cw, ih = (wi / cw) % ch, id = wi / (cw * ch);
    int d0 = id * stride; if (d0 > D - P) d0 = D - P;
    int h0 = ih * stride; if (h0 > H - P) h0 = H - P;
    int w0 = iw * stride; if (w0 > W - P) w0 = W - P;
    win[idx] = vol[((((int64_t)(d0 + i)) * H + (h0 + j)) * W + (w0 + k)) * C + c];
}

// One thread per volume voxel: gathers every covering window in d-major, h, w order.
__global__ __launch_bounds__(256) void sw_blend_kernel(const float* __restrict__ wl, float* __restrict__ out, int D, int H,
                                                       int W, int K, int P, int stride, int cd, int ch, int cw,
                                                       float inv2s2) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v >= (int64_t)D * H * W) return;
    const int w = (int)(v % W), h = (int)((v / W) % H), d = (int)(v / ((int64_t)W * H));
    const float m = 0.5f * (P - 1);
    const bool even = (K & 1) == 0;
    float acc[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) acc[k] = 0.f;
    float wsum = 0.f;
    for (int id = 0; id < cd; ++id) {
        int d0 = id * stride; if (d0 > D - P) d0 = D - P;
        if (d < d0 || d >= d0 + P) continue;
        const float fd = (d - d0) - m;
        for (int ih = 0; ih < ch; ++ih) {
            int h0 = ih * stride; if (h0 > H - P) h0 = H - P;
            if (h < h0 || h >= h0 + P) continue;
            const float fh = (h - h0) - m;
            for (int iw = 0; iw < cw; ++iw) {
                int w0 = iw * stride; if (w0 > W - P) w0 = W - P;
                if (w < w0 || w >= w0 + P) continue;
                const float fw = (w - w0) - m;
                const float g = expf(-(fd * fd + fh * fh + fw * fw) * inv2s2);
                const int wi = (id * ch + ih) * cw + iw;
                const float* p = wl + ((((int64_t)wi * P + (d - d0)) * P + (h - h0)) * P + (w - w0)) * K;
                if (even) {   // a voxel's K floats start on an 8-byte boundary: half as many load instructions
                    const float2* p2 = reinterpret_cast<const float2*>(p);
#pragma unroll
                    for (int k = 0; k < 8; ++k)
                        if (2 * k < K) {
                            const float2 t = p2[k];
                            acc[2 * k] = fmaf(g, t.x, acc[2 * k]);
                            acc[2 * k + 1] = fmaf(g, t.y, acc[2 * k + 1]);
                        }
                } else {
#pragma unroll
                    for (int k = 0; k < 16; ++k)
                        if (k < K) acc[k] = fmaf(g, p[k], acc[k]);
                }
                wsum += g;
            }
        }
    }
    if (even) {
        float2* o2 = reinterpret_cast<float2*>(out + v * K);
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (2 * k < K) o2[k] = make_float2(acc[2 * k] / wsum, acc[2 * k + 1] / wsum);
    } else {
#pragma unroll
        for (int k = 0; k < 16; ++k)
            if (k < K) out[v * K + k] = acc[k] / wsum;
    }
}

}  // namespace lamp

extern "C" int32_t lamp_sliding_window_count(int32_t D, int32_t H, int32_t W, int32_t patch, float overlap) {
    if (patch < 1 || D < patch || H < patch || W < patch || !(overlap >= 0.f) || !(overlap < 1.f)) return 0;
    const int s = sw_stride(patch, overlap);
    if (s < 1) return 0;
    return sw_count1(D, patch, s) * sw_count1(H, patch, s) * sw_count1(W, patch, s);
}

extern "C" size_t lamp_sliding_window_workspace_bytes(const lamp_unet_desc* pd, int32_t D, int32_t H, int32_t W) {
    if (unet_desc_ok(pd) != LAMP_OK) return 0;
    const int64_t per = (int64_t)pd->d * pd->h * pd->w;
    return align_up((size_t)pd->n * per * pd->in_ch * esize(pd->dtype)) +
           align_up((size_t)pd->n * per * pd->classes * sizeof(float)) + lamp_unet_workspace_bytes(pd, 0) + 512;
}

extern "C" lamp_status lamp_sliding_window_fwd(const lamp_unet_desc* pd, const void* const* params, const void* vol,
                                               int32_t D, int32_t H, int32_t W, float overlap, float sigma_scale,
                                               float* out, void* ws, size_t ws_bytes, void* stream) {
    lamp_status st = unet_desc_ok(pd);
    if (st != LAMP_OK) return st;
    if (!params || !vol || !out) return LAMP_ERR_NULL;
    const int P = pd->d;
    if (pd->h != P || pd->w != P) return LAMP_ERR_SHAPE;
    const int cnt = lamp_sliding_window_count(D, H, W, P, overlap);
    if (cnt < 1 || cnt != pd->n || !(sigma_scale > 0.f)) return LAMP_ERR_SHAPE;
    if (!ws || ws_bytes < lamp_sliding_window_workspace_bytes(pd, D, H, W)) return LAMP_ERR_WORKSPACE;
    if (!aligned16(ws) || !aligned16(vol)) return LAMP_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    const int stride = sw_stride(P, overlap);
    const int cd = sw_count1(D, P, stride), ch = sw_count1(H, P, stride), cw = sw_count1(W, P, stride);
    const int64_t per = (int64_t)P * P * P;
    Carver cv(ws, ws_bytes);
    void* win = cv.take((size_t)cnt * per * pd->in_ch * esize(pd->dtype));
    float* wl = (float*)cv.take((size_t)cnt * per * pd->classes * sizeof(float));
    const size_t ub = lamp_unet_workspace_bytes(pd, 0);
    void* uws = cv.take(ub);
    if (!cv.ok()) return LAMP_ERR_WORKSPACE;
    const int64_t tot = (int64_t)cnt * per * pd->in_ch;
    if (pd->dtype == LAMP_BF16)
        hipLaunchKernelGGL((sw_gather_kernel<bf16_t>), dim3(cdiv(tot, 256)), dim3(256), 0, s, (const bf16_t*)vol,
                           (bf16_t*)win, D, H, W, pd->in_ch, P, stride, cd, ch, cw);
    else
        hipLaunchKernelGGL((sw_gather_kernel<float>), dim3(cdiv(tot, 256)), dim3(256), 0, s, (const float*)vol, (float*)win,
                           D, H, W, pd->in_ch, P, stride, cd, ch, cw);
    LAMP_CHECK_LAUNCH();
    if ((st = lamp_unet_fwd(pd, params, win, wl, uws, ub, stream)) != LAMP_OK) return st;
    const float sg = sigma_scale * P;
    hipLaunchKernelGGL(sw_blend_kernel, dim3(cdiv((int64_t)D * H * W, 256)), dim3(256), 0, s, wl, out, D, H, W, pd->classes,
                       P, stride, cd, ch, cw, 0.5f / (sg * sg));
    LAMP_CHECK_LAUNCH();
    return LAMP_OK;
}
