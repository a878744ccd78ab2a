// Register-resident MFMA-only loop: what the matrix instruction of the attention kernels sustains
// on this machine when nothing else competes with it (see grat_probe.h).
#include <hip/hip_runtime.h>

#include "grat_probe.h"

namespace grat {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

template <bool F16>
__global__ __launch_bounds__(256) void mfma_probe_kernel(long long* sink, int iters, float one) {
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    // Operands: small integers that differ from lane to lane and element to element (what the
    // matrix pipe draws, and with it the clock the chip holds, depends on how the data toggles;
    // constant operands would flatter it).  `one` arrives as an argument so that nothing of the
    // loop can be folded at compile time.
    const int lane = threadIdx.x & 63;
    bf16x8 ab, bb;
    f16x8 ah, bh;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float a = one * (float)((lane * 37 + e * 11 + 5) % 9 - 4);
        const float b = one * (float)((lane * 53 + e * 17 + 2) % 9 - 4);
        ab[e] = (__bf16)a; bb[e] = (__bf16)b;
        ah[e] = (_Float16)a; bh[e] = (_Float16)b;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (F16) acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh, acc[j & 3], 0, 0, 0);
            else acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ab, bb, acc[j & 3], 0, 0, 0);
        }
    }
    long long s = 0;   // every accumulator value is an integer below 2^24: the sum is exact
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += (long long)acc[i][r];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace
}  // namespace grat

extern "C" grat_status grat_probe_mfma(grat_dtype dtype, int64_t* d_sink, int32_t blocks, int32_t iters,
                                       void* hip_stream) {
    if (!d_sink) return GRAT_ERR_NULL;
    if (blocks < 1 || blocks > 65536 || iters < 1 || iters > 4096) return GRAT_ERR_BAD_DIMS;
    if (dtype != GRAT_BF16 && dtype != GRAT_F16) return GRAT_ERR_UNSUPPORTED;
    hipStream_t stream = (hipStream_t)hip_stream;
    if (dtype == GRAT_F16)
        hipLaunchKernelGGL(grat::mfma_probe_kernel<true>, dim3(blocks), dim3(256), 0, stream, (long long*)d_sink, iters, 1.0f);
    else
        hipLaunchKernelGGL(grat::mfma_probe_kernel<false>, dim3(blocks), dim3(256), 0, stream, (long long*)d_sink, iters, 1.0f);
    return hipGetLastError() == hipSuccess ? GRAT_OK : GRAT_ERR_HIP;
}
