// Register-resident MFMA-only loop: what the matrix instruction of the attention kernels sustains
// on this machine when nothing else competes with it (see grat_probe.h).
#include <hip/hip_runtime.h>

#include <cstdint>

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
    // Operands change from lane to lane, element to element and instruction to instruction, and six
    // of the eight instructions of an iteration work on full 8-bit significands: what the matrix
    // pipe draws, and with it the clock the chip holds, depends on how the data toggles; constant
    // or narrow operands would flatter it.  Accumulators 0..2 take  A_v B_v  and then  A_v (-B_v)
    // (every partial sum is a multiple of 1/256 below 2^24, so they return to exactly 0);
    // accumulator 3 takes two products of small integers per iteration and keeps the count.
    // `one` arrives as an argument so that nothing of the loop can be folded at compile time.
    const int lane = threadIdx.x & 63;
    bf16x8 ab[4], bb[5], nb[3];
    f16x8 ah[4], bh[5], nh[3];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
#pragma unroll
        for (int v = 0; v < 3; ++v) {
            const uint32_t ha = (uint32_t)(lane * 73 + e * 151 + v * 199 + 17) * 2654435761u;
            const uint32_t hb = (uint32_t)(lane * 89 + e * 131 + v * 211 + 29) * 2246822519u;
            const float a = one * (float)((int)(ha >> 24) - 128) * 0.0625f;
            const float b = one * (float)((int)(hb >> 24) - 128) * 0.0625f;
            ab[v][e] = (__bf16)a; bb[v][e] = (__bf16)b; nb[v][e] = (__bf16)(-b);
            ah[v][e] = (_Float16)a; bh[v][e] = (_Float16)b; nh[v][e] = (_Float16)(-b);
        }
        const float ia = one * (float)((lane * 37 + e * 11 + 5) % 9 - 4);
        const float ib0 = one * (float)((lane * 53 + e * 17 + 2) % 9 - 4);
        const float ib1 = one * (float)((lane * 57 + e * 13 + 7) % 9 - 4);
        ab[3][e] = (__bf16)ia; bb[3][e] = (__bf16)ib0; bb[4][e] = (__bf16)ib1;
        ah[3][e] = (_Float16)ia; bh[3][e] = (_Float16)ib0; bh[4][e] = (_Float16)ib1;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int v = j & 3;
            if (F16) {
                const f16x8 b = v == 3 ? bh[3 + (j >> 2)] : (j < 4 ? bh[v] : nh[v]);
                acc[v] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah[v], b, acc[v], 0, 0, 0);
            } else {
                const bf16x8 b = v == 3 ? bb[3 + (j >> 2)] : (j < 4 ? bb[v] : nb[v]);
                acc[v] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ab[v], b, acc[v], 0, 0, 0);
            }
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
