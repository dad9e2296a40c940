// Cross-file internal entry points of liblamp (host side).  Not part of the ABI.
#pragma once
#include "common.h"

namespace lamp {

// ---- api.hip --------------------------------------------------------------------------------
// Value of `key` in the LAMP_TUNE environment variable ("key=value,key=value"; a bare key means 1), else dflt.
int tune(const char* key, int dflt);
// Raises a kernel's dynamic-LDS limit once per (device, kernel); thread-safe.
lamp_status ensure_dyn_lds(const void* fn, int bytes);

// ---- norm.hip -------------------------------------------------------------------------------
// Number of row chunks the stand-alone statistics pass uses for a tensor of `v` voxels per sample.
int stats_chunks(int64_t v);
// Bytes of workspace for the stand-alone statistics pass (partials [N][chunks][C][2] fp32).
size_t stats_ws_bytes(const lamp_tensor_desc* zd);
lamp_status launch_splitk_reduce(const float* zpart, int S, const lamp_tensor_desc* zd, void* z, float eps, float* stats,
                                 void* ws, size_t ws_bytes, hipStream_t s, void* z2 = nullptr, int ldz2 = 0, int zsplit = 0);
// Two-kernel statistics of z: writes stats[N][C][2] = (mean, rstd).
lamp_status launch_stats(const lamp_tensor_desc* zd, const void* z, float eps, float* stats,
                         void* ws, size_t ws_bytes, hipStream_t s);
// Combine per-part (sum, sumsq) fp32 partials [N][parts][C][2] with per-part voxel counts (int32;
// cnt[parts], the same for every sample, or cnt[N][parts] when counts_per_sample) into
// stats[N][C][2]; fp64 pairwise merging.
lamp_status launch_stats_finalize(const float* partials, const int32_t* counts, int parts, int N, int C,
                                  float eps, float* stats, hipStream_t s, bool counts_per_sample = false);

// Per-tile partials (sum g, sum g*z) of a data-gradient epilogue to sums[N][C][2] = (sum g, sum g*zhat); fp64, fixed order.
lamp_status launch_bsum_finalize(const float* partial, int parts, int N, int C, const float* zstats, float* sums, hipStream_t s);
// The element-wise half of the InstanceNorm + ReLU backward for given sums[N][C][2] (and dgamma / dbeta from them).
lamp_status launch_inorm_bwd_apply(const lamp_tensor_desc* dyd, const void* dy, const lamp_tensor_desc* zd, const void* z,
                                   const float* stats, const float* gamma, const float* beta, const float* sums,
                                   const lamp_tensor_desc* dzd, void* dz, float* dgamma, float* dbeta, float beta_acc,
                                   hipStream_t s);

// ---- reduce.hip -----------------------------------------------------------------------------
// out[o] = beta*out[o] + sum_s part[s][o], s in fixed order, fp64 accumulation.
// ---- repacked conv weights prepared ahead of the calls that use them (network entry points) ----
// kind: 0 tiled kernel with the 4-deep tile, 1 with the 8-deep tile (kh-major taps); -1: the shape does not take a
// matrix-core path.
struct RepackJob { const void* w; void* wp; int Cout, Cin, dgrad, kind; };
struct RepackTable { int n; RepackJob e[64]; };
// two_out: the conv writes a two-part tensor (then a batch of small volumes is not packed into one volume).
int conv_repack_kind(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd, bool two_out = false);
size_t conv_repack_bytes(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd);
lamp_status launch_repack_batch(const RepackJob* jobs, int n, hipStream_t s);
// The table the calling thread's conv calls consult (weight pointer + direction + kind must match);
// nullptr outside a network entry point.
void set_repack_table(const RepackTable* t);
const bf16_t* find_prepacked(const void* w, bool dgrad, int kind, int Cout, int Cin);
const bf16_t* device_zero16();  // 16 zero bytes on the current device, nullptr on failure
lamp_status launch_reduce_partials(const float* part, int S, int64_t O, float* out, float beta, hipStream_t s);
// Column sums of a [rows, C] tensor with row stride ld: out[c] = beta*out[c] + sum_r t[r][c].
size_t colsum_ws_bytes(int64_t rows, int C);
lamp_status launch_colsum(const void* t, int dtype, int64_t rows, int C, int ld, float* out, float beta,
                          void* ws, size_t ws_bytes, hipStream_t s);

// ---- se.hip ---------------------------------------------------------------------------------
// a[i] += b[i] over numel elements of the storage dtype (dense tensors).
lamp_status launch_add_inplace(void* a, const void* b, int64_t numel, int dtype, hipStream_t s);

// ---- head.hip -------------------------------------------------------------------------------
// lamp_head_ce with the mean taken over norm_count voxels (0: the call's own) and the loss added to
// *loss when loss_beta == 1.
lamp_status head_ce_run(const lamp_tensor_desc* xd, const void* x, const lamp_norm_in* xnorm, const void* wh,
                        const float* bh, int classes, const int32_t* labels, float* logits, float* loss,
                        const lamp_tensor_desc* dxd, void* dx, float* dwh, float* dbh, float beta, int64_t norm_count,
                        float loss_beta, void* ws, size_t ws_bytes, void* stream);

// ---- conv3d_mfma.hip ------------------------------------------------------------------------
// Matrix-core implicit-GEMM paths; each returns LAMP_ERR_UNSUPPORTED when the shape is not one
// they serve, and the caller falls back to the generic kernels.
// InstanceNorm + ReLU of a raw conv output z (statistics and affine parameters in xnorm, all channels) fused with
// the 2x2x2 max-pool of the result: writes the activated tensor to yfull (channel stride ldyf) and the pooled one to y.
lamp_status inorm_relu_maxpool2(const lamp_tensor_desc* xd, const void* z, const lamp_norm_in* xnorm, void* yfull, int ldyf,
                                const lamp_tensor_desc* yd, void* y, hipStream_t s);
bool mfma_conv_supported(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd, const lamp_norm_in* xnorm,
                         const float* bias);
size_t mfma_conv_ws_bytes(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd, int want_stats);
// Two-part tensors: a channel concat that is never materialised.  x2: second input tensor holding the
// input channels from x_c1 on (same channel stride as x, x_c1 % 16 == 0); z2: second output tensor
// receiving the output channels from z_c1 on (channel stride ldz2, z_c1 % 32 == 0).  With parts the
// tiled kernel is used whatever the shape.
struct ConvParts { const void* x2; int x_c1; void* z2; int z_c1, ldz2; };
// Data gradient that also takes the two sums of the InstanceNorm + ReLU backward of the layer below: z = that layer's
// raw conv output (voxels, channels and channel stride of the tensor the data gradient writes), stats / gamma / beta
// its statistics and affine parameters, sums_out [N][C][2] = (sum g, sum g*zhat) with g = [u > 0] * dx.
struct ConvBsum { const void* z; const float* stats; const float* gamma; const float* beta; float* sums_out; };
bool mfma_bsum_supported(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd);
size_t mfma_bsum_ws_bytes(const lamp_tensor_desc* xd, const lamp_tensor_desc* zd);
lamp_status mfma_conv_fwd(const lamp_tensor_desc* xd, const void* x, const void* w, bool dgrad,
                          const lamp_tensor_desc* zd, void* z, float* stats_out, float eps,
                          void* ws, size_t ws_bytes, hipStream_t s, const ConvParts* parts = nullptr,
                          const float* bias = nullptr, const lamp_norm_in* xnorm = nullptr, const ConvBsum* bsum = nullptr);
bool mfma_wgrad_supported(const lamp_tensor_desc* xd, const lamp_tensor_desc* dzd, const lamp_norm_in* xnorm);
size_t mfma_wgrad_ws_bytes(const lamp_tensor_desc* xd, const lamp_tensor_desc* dzd);
lamp_status mfma_wgrad(const lamp_tensor_desc* xd, const void* x, const lamp_tensor_desc* dzd, const void* dz,
                       float* dw, float beta, void* ws, size_t ws_bytes, hipStream_t s, const void* x2 = nullptr,
                       int x_c1 = 0);

// ---- convtr_mfma.hip ------------------------------------------------------------------------
bool mfma_convtr_supported(const lamp_tensor_desc* xd, const lamp_tensor_desc* yd, const lamp_norm_in* xnorm);
size_t mfma_convtr_ws_bytes(const lamp_tensor_desc* xd, const lamp_tensor_desc* yd);
lamp_status mfma_convtr_fwd(const lamp_tensor_desc* xd, const void* x, const void* wt, const float* bias,
                            const lamp_tensor_desc* yd, void* y, void* ws, size_t ws_bytes, hipStream_t s);
bool mfma_convtr_dgrad_supported(const lamp_tensor_desc* xd, const lamp_tensor_desc* dyd, const lamp_tensor_desc* dxd);
lamp_status mfma_convtr_dgrad(const lamp_tensor_desc* xd, const void* wt, const lamp_tensor_desc* dyd, const void* dy,
                              const lamp_tensor_desc* dxd, void* dx, hipStream_t s);

bool mfma_convtr_wgrad_supported(const lamp_tensor_desc* xd, const lamp_tensor_desc* dyd, const lamp_norm_in* xnorm);
size_t mfma_convtr_wgrad_ws_bytes(const lamp_tensor_desc* xd, const lamp_tensor_desc* dyd);
lamp_status mfma_convtr_wgrad(const lamp_tensor_desc* xd, const void* x, const lamp_tensor_desc* dyd, const void* dy,
                              float* dwt, float beta, void* ws, size_t ws_bytes, hipStream_t s);

}  // namespace lamp
