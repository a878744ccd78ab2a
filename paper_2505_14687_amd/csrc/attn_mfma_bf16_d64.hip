// One slice of the MFMA attention kernel's instantiations (element type x head_dim), in a
// translation unit of its own so that the slices compile side by side.
#include "attn_mfma.h"

namespace grat {

hipError_t launch_mfma_bf16_d64(const AttnParams& p, int mode, hipStream_t stream) {
    return launch_by_tile<false, 64>(p, mode, stream);
}

}  // namespace grat
