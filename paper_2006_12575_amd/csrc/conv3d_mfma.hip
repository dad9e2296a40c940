// Matrix-core (MFMA) implicit-GEMM convolution kernels for gfx950.
#include "internal.h"

namespace lamp {

bool mfma_conv_supported(const lamp_tensor_desc*, const lamp_tensor_desc*, const lamp_norm_in*, const float*) { return false; }
size_t mfma_conv_ws_bytes(const lamp_tensor_desc*, const lamp_tensor_desc*, int) { return 0; }
lamp_status mfma_conv_fwd(const lamp_tensor_desc*, const void*, const void*, bool, const lamp_tensor_desc*, void*, float*,
                          float, void*, size_t, hipStream_t) { return LAMP_ERR_UNSUPPORTED; }
bool mfma_wgrad_supported(const lamp_tensor_desc*, const lamp_tensor_desc*, const lamp_norm_in*) { return false; }
size_t mfma_wgrad_ws_bytes(const lamp_tensor_desc*, const lamp_tensor_desc*) { return 0; }
lamp_status mfma_wgrad(const lamp_tensor_desc*, const void*, const lamp_tensor_desc*, const void*, float*, float, void*,
                       size_t, hipStream_t) { return LAMP_ERR_UNSUPPORTED; }

}  // namespace lamp
