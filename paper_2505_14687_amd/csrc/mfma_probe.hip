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

// small integer -4..4 for (lane, element, fragment v, which = 0 for A / 1 for B)
__device__ __forceinline__ float small_int(int lane, int e, int v, int which) {
    return (float)((lane * (37 + 16 * which + 2 * v) + e * (11 + 6 * which) + 5 + 3 * v - 3 * which) % 9 - 4);
}

// n / 64 with n an integer of at most 8 significant bits, distributed roughly like 64 N(0,1)
// (sum of four hash bytes, centred and scaled)
__device__ __forceinline__ float normal_like(int lane, int e, int v, int which) {
    uint32_t h = (uint32_t)(lane * 73 + e * 151 + v * 199 + which * 977 + 17) * 2654435761u;
    h ^= (h >> 15) * 2246822519u;
    const int sum = (int)(h & 255) + (int)((h >> 8) & 255) + (int)((h >> 16) & 255) + (int)(h >> 24);   // 0..1020
    const int n = ((sum - 510) * 111) / 256;   // |n| <= 221
    return (float)n * (1.f / 64.f);
}

template <bool F16>
__global__ __launch_bounds__(256) void mfma_probe_kernel(long long* sink, int iters, int data, float one) {
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    // Fragments: accumulator v takes  A_v B_v  and then  A_v B'_v  in every iteration.
    //   data 0: all ones, B' = B;  data 1: small integers, B' = B (the accumulators count up);
    //   data 2: v < 3: 8-bit significands spread like N(0,1), B' = -B - every partial sum is a
    //           multiple of 1/4096 below 2^24, so these accumulators return to exactly 0;
    //           v = 3: small integers, B' = B, keeps the count.
    // (`one` arrives as an argument so that nothing of the loop can be folded at compile time)
    const int lane = threadIdx.x & 63;
    bf16x8 ab[4], bb[4], cb[4];
    f16x8 ah[4], bh[4], ch[4];
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float a, b, c;
            if (data == 0) {
                a = b = c = 1.f;
            } else if (data == 1 || v == 3) {
                a = small_int(lane, e, v, 0);
                b = c = small_int(lane, e, v, 1);
            } else {
                a = normal_like(lane, e, v, 0);
                b = normal_like(lane, e, v, 1);
                c = -b;
            }
            a *= one; b *= one; c *= one;
            ab[v][e] = (__bf16)a; bb[v][e] = (__bf16)b; cb[v][e] = (__bf16)c;
            ah[v][e] = (_Float16)a; bh[v][e] = (_Float16)b; ch[v][e] = (_Float16)c;
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int v = j & 3;
            if (F16) acc[v] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah[v], j < 4 ? bh[v] : ch[v], acc[v], 0, 0, 0);
            else acc[v] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ab[v], j < 4 ? bb[v] : cb[v], acc[v], 0, 0, 0);
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

extern "C" grat_status grat_probe_mfma(grat_dtype dtype, int32_t data, int64_t* d_sink, int32_t blocks,
                                       int32_t iters, void* hip_stream) {
    if (!d_sink) return GRAT_ERR_NULL;
    if (blocks < 1 || blocks > 65536 || iters < 1 || iters > 4096 || data < 0 || data > 2) return GRAT_ERR_BAD_DIMS;
    if (dtype != GRAT_BF16 && dtype != GRAT_F16) return GRAT_ERR_UNSUPPORTED;
    hipStream_t stream = (hipStream_t)hip_stream;
    if (dtype == GRAT_F16)
        hipLaunchKernelGGL(grat::mfma_probe_kernel<true>, dim3(blocks), dim3(256), 0, stream, (long long*)d_sink,
                           iters, data, 1.0f);
    else
        hipLaunchKernelGGL(grat::mfma_probe_kernel<false>, dim3(blocks), dim3(256), 0, stream, (long long*)d_sink,
                           iters, data, 1.0f);
    return hipGetLastError() == hipSuccess ? GRAT_OK : GRAT_ERR_HIP;
}
