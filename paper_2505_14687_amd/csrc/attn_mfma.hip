// Dispatch of the MFMA attention path to the instantiation slices (see attn_mfma.h for the kernel).
#include "grat_common.h"

namespace grat {

hipError_t launch_mfma_bf16_d128(const AttnParams& p, int mode, hipStream_t stream);
hipError_t launch_mfma_bf16_d64(const AttnParams& p, int mode, hipStream_t stream);
hipError_t launch_mfma_f16_d128(const AttnParams& p, int mode, hipStream_t stream);
hipError_t launch_mfma_f16_d64(const AttnParams& p, int mode, hipStream_t stream);

// f16: the elements are IEEE half instead of bfloat16; head_dim 128 or 64 (checked by the caller).
hipError_t launch_attn_bf16(const AttnParams& p, int mode, bool f16, int head_dim, hipStream_t stream) {
    if (head_dim == 64) return f16 ? launch_mfma_f16_d64(p, mode, stream) : launch_mfma_bf16_d64(p, mode, stream);
    return f16 ? launch_mfma_f16_d128(p, mode, stream) : launch_mfma_bf16_d128(p, mode, stream);
}

}  // namespace grat
