// Block-list builder: for every query group the ascending list of attendable KV group ids
// (Sec. 3.2: Eq. 5-6 / 12-13 surrounding blocks, Eq. 7-8 / 14-15 criss-cross regions).
//
// One 64-lane wavefront per query group scans all candidate KV groups in ascending id order,
// 64 at a time; a ballot plus a prefix popcount compacts the survivors, so the output order
// is ascending by construction and any predicate on group coordinates fits.
#include "grat_common.h"

namespace grat {

struct ListParams {
    int32_t G[3];
    int32_t radius[3];
    int32_t num_groups;
    int32_t ndim;
    int32_t pattern;
    int32_t max_kv;
    int32_t* kv_count;
    int32_t* kv_index;
};

__global__ __launch_bounds__(64) void build_block_lists_kernel(ListParams p) {
    const int gamma = blockIdx.x;
    const int lane = threadIdx.x;
    const int G12 = p.G[1] * p.G[2];
    const int q0 = gamma / G12, q1 = (gamma / p.G[2]) % p.G[1], q2 = gamma % p.G[2];
    int32_t* row = p.kv_index + (int64_t)gamma * p.max_kv;
    int cnt = 0;
    for (int base = 0; base < p.num_groups; base += 64) {
        const int cand = base + lane;
        bool ok = false;
        if (cand < p.num_groups) {
            const int k0 = cand / G12, k1 = (cand / p.G[2]) % p.G[1], k2 = cand % p.G[2];
            const int d0 = abs(k0 - q0), d1 = abs(k1 - q1), d2 = abs(k2 - q2);
            if (p.pattern == GRAT_BLOCK) {
                ok = d0 <= p.radius[0] && d1 <= p.radius[1] && d2 <= p.radius[2];
            } else if (p.pattern == GRAT_DENSE) {
                ok = true;
            } else {
                // axes beyond ndim have extent 1 and always match: count real axes only
                const int differ = (d0 != 0) + (d1 != 0) + (d2 != 0);
                ok = p.pattern == GRAT_CROSS ? differ <= 1 : differ <= p.ndim - 1;
            }
        }
        const unsigned long long m = __ballot(ok);
        if (ok) {
            const int pos = cnt + __popcll(m & ((1ull << lane) - 1ull));
            if (pos < p.max_kv) row[pos] = cand;
        }
        cnt += __popcll(m);
    }
    for (int i = cnt + lane; i < p.max_kv; i += 64) row[i] = -1;
    if (lane == 0) p.kv_count[gamma] = cnt;
}

// Checks lists against the format above: one wave per query group; violations are OR-ed into
// *status (cleared by a one-thread launch ahead of this one, so no host-side memset is involved).
__global__ void clear_status_kernel(int32_t* status) { *status = 0; }
__global__ __launch_bounds__(64) void validate_block_lists_kernel(const int32_t* kv_count, const int32_t* kv_index,
                                                                  int32_t num_groups, int32_t max_kv, int32_t* status) {
    const int gamma = blockIdx.x, lane = threadIdx.x;
    const int cnt = kv_count[gamma];
    int bad = (cnt < 1 || cnt > max_kv) ? GRAT_LIST_BAD_COUNT : 0;
    const int used = min(max(cnt, 0), max_kv);
    const int32_t* row = kv_index + (int64_t)gamma * max_kv;
    for (int i = lane; i < max_kv; i += 64) {
        const int v = row[i];
        if (i < used) {
            if (v < 0 || v >= num_groups) bad |= GRAT_LIST_BAD_ENTRY;
        } else if (v != -1) {
            bad |= GRAT_LIST_BAD_PADDING;
        }
    }
    if (bad) atomicOr(status, bad);
}

hipError_t launch_validate_block_lists(const Geometry& geo, const int32_t* d_kv_count, const int32_t* d_kv_index,
                                       int32_t max_kv, int32_t* d_status, hipStream_t stream) {
    hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, stream, d_status);
    hipLaunchKernelGGL(validate_block_lists_kernel, dim3(geo.num_groups), dim3(64), 0, stream, d_kv_count, d_kv_index,
                       geo.num_groups, max_kv, d_status);
    return hipGetLastError();
}

hipError_t launch_build_block_lists(const Geometry& geo, int ndim, grat_pattern pattern,
                                    const int32_t radius[3], int32_t* d_kv_count,
                                    int32_t* d_kv_index, int32_t max_kv, hipStream_t stream) {
    ListParams p;
    for (int k = 0; k < 3; ++k) { p.G[k] = geo.G[k]; p.radius[k] = radius[k]; }
    p.num_groups = geo.num_groups;
    p.ndim = ndim;
    p.pattern = (int32_t)pattern;
    p.max_kv = max_kv;
    p.kv_count = d_kv_count;
    p.kv_index = d_kv_index;
    hipLaunchKernelGGL(build_block_lists_kernel, dim3(geo.num_groups), dim3(64), 0, stream, p);
    return hipGetLastError();
}

}  // namespace grat
