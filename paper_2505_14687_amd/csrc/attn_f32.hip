// fp32 attention (grouped and dense): plain vector-ALU kernel, one query per lane.
//
// Sec. 3.1 Eq. 1 restricted to the attendable KV groups of Sec. 3.2.  This is the precision
// path (inputs, scores, softmax and accumulation all fp32); throughput is not its purpose.
// One 64-lane wavefront owns up to 64 queries of one group; K/V rows of the attendable groups
// are staged through LDS 32 tokens at a time and every lane reads them as broadcasts.
// Group dims need not divide the grid (Eq. 2-4 are floor divisions): a group at the far border
// is the part of its box that lies inside the grid, and its tokens are enumerated over that part.
#include "grat_common.h"

namespace grat {

constexpr int kF32Keys = 32;   // KV tokens staged per LDS tile

template <int D, bool DENSE>
__global__ __launch_bounds__(64) void attn_f32_kernel(AttnParams p) {
    __shared__ float sK[kF32Keys][D];
    __shared__ float sV[kF32Keys][D];

    const int lane = threadIdx.x;
    const int tile = xcd_contiguous_tile(blockIdx.x, p.total_tiles);
    if (tile >= p.total_tiles) return;

    const Geometry& geo = p.geo;
    const int tiles_per_head = DENSE ? p.q_tiles : geo.num_groups * p.q_tiles;
    const int bh = tile / tiles_per_head;
    const int t_in_head = tile % tiles_per_head;
    const int64_t head_off = (int64_t)(bh / p.heads) * p.stride_b + (int64_t)(bh % p.heads) * p.stride_h;
    const float* Qh = (const float*)p.Q + head_off;
    const float* Kh = (const float*)p.K + head_off;
    const float* Vh = (const float*)p.V + head_off;
    float* Oh = (float*)p.O + (int64_t)(bh / p.heads) * p.o_stride_b + (int64_t)(bh % p.heads) * p.o_stride_h;

    const int T12 = geo.T[1] * geo.T[2];
    const int G12 = geo.G[1] * geo.G[2];

    // A group as its first token row and the extents of its box inside the grid.
    struct Box { int origin, v1, v2, tokens; };
    auto group_box = [&](int gid) {
        const int p0 = gid / G12, p1 = (gid / geo.G[2]) % geo.G[1], p2 = gid % geo.G[2];
        const int v0 = min(geo.g[0], geo.T[0] - p0 * geo.g[0]);
        Box b;
        b.v1 = min(geo.g[1], geo.T[1] - p1 * geo.g[1]);
        b.v2 = min(geo.g[2], geo.T[2] - p2 * geo.g[2]);
        b.origin = p0 * geo.g[0] * T12 + p1 * geo.g[1] * geo.T[2] + p2 * geo.g[2];
        b.tokens = v0 * b.v1 * b.v2;
        return b;
    };
    // token row of the t-th token of a group (last axis fastest inside its box)
    auto token_row = [&](const Box& b, int t) {
        return b.origin + (t / (b.v1 * b.v2)) * T12 + ((t / b.v2) % b.v1) * geo.T[2] + t % b.v2;
    };

    int gamma = 0, q_row, n_lists, list_tokens;
    bool q_valid;
    if (DENSE) {
        q_row = t_in_head * 64 + lane;
        q_valid = q_row < p.n_tokens;
        n_lists = 1;
        list_tokens = p.n_tokens;
    } else {
        gamma = t_in_head / p.q_tiles;
        const Box qb = group_box(gamma);
        if ((t_in_head % p.q_tiles) * 64 >= qb.tokens) return;   // a border group with fewer query tiles
        const int t = (t_in_head % p.q_tiles) * 64 + lane;
        q_valid = t < qb.tokens;
        q_row = token_row(qb, q_valid ? t : 0);
        n_lists = min(max(p.kv_count[gamma], 0), p.max_kv);   // (forced into range: a bad list never reads outside the tensors)
        list_tokens = 0;   // per listed group, below
    }
    if (!q_valid && DENSE) q_row = p.n_tokens - 1;

    float q[D], o[D];
    {
        const float4* src = (const float4*)(Qh + (int64_t)q_row * p.stride_n);
#pragma unroll
        for (int c = 0; c < D / 4; ++c) {
            const float4 v = src[c];
            q[4 * c] = v.x; q[4 * c + 1] = v.y; q[4 * c + 2] = v.z; q[4 * c + 3] = v.w;
        }
#pragma unroll
        for (int c = 0; c < D; ++c) o[c] = 0.f;
    }
    float m = -INFINITY, l = 0.f;

    for (int li = 0; li < n_lists; ++li) {
        Box kb{0, 1, 1, 0};
        if (!DENSE) {
            kb = group_box(min(max(p.kv_index[(int64_t)gamma * p.max_kv + li], 0), p.geo.num_groups - 1));
            list_tokens = kb.tokens;
        }
        for (int t0 = 0; t0 < list_tokens; t0 += kF32Keys) {
            const int n_valid = min(kF32Keys, list_tokens - t0);
            __syncthreads();
            // stage K and V rows: D/4 float4 per row, 64 lanes
            for (int c = lane; c < kF32Keys * (D / 4); c += 64) {
                const int kk = c / (D / 4), col = c % (D / 4);
                if (kk < n_valid) {
                    const int row = DENSE ? t0 + kk : token_row(kb, t0 + kk);
                    const int64_t off = (int64_t)row * p.stride_n + 4 * col;
                    *(float4*)&sK[kk][4 * col] = *(const float4*)(Kh + off);
                    *(float4*)&sV[kk][4 * col] = *(const float4*)(Vh + off);
                }
            }
            __syncthreads();

            float s[kF32Keys];
            float tile_max = -INFINITY;
#pragma unroll
            for (int kk = 0; kk < kF32Keys; ++kk) {
                float acc = 0.f;
                if (kk < n_valid) {
#pragma unroll
                    for (int c = 0; c < D; c += 4) {
                        const float4 kv = *(const float4*)&sK[kk][c];
                        acc = fmaf(q[c], kv.x, acc);
                        acc = fmaf(q[c + 1], kv.y, acc);
                        acc = fmaf(q[c + 2], kv.z, acc);
                        acc = fmaf(q[c + 3], kv.w, acc);
                    }
                    acc *= p.scale_log2;
                    tile_max = fmaxf(tile_max, acc);
                } else {
                    acc = -INFINITY;
                }
                s[kk] = acc;
            }
            const float m_new = fmaxf(m, tile_max);
            const float alpha = exp2f(m - m_new);   // first tile: exp2(-inf) = 0
            l *= alpha;
#pragma unroll
            for (int c = 0; c < D; ++c) o[c] *= alpha;
#pragma unroll
            for (int kk = 0; kk < kF32Keys; ++kk) {
                if (kk < n_valid) {
                    const float w = exp2f(s[kk] - m_new);
                    l += w;
#pragma unroll
                    for (int c = 0; c < D; c += 4) {
                        const float4 vv = *(const float4*)&sV[kk][c];
                        o[c] = fmaf(w, vv.x, o[c]);
                        o[c + 1] = fmaf(w, vv.y, o[c + 1]);
                        o[c + 2] = fmaf(w, vv.z, o[c + 2]);
                        o[c + 3] = fmaf(w, vv.w, o[c + 3]);
                    }
                }
            }
            m = m_new;
        }
    }

    if (q_valid) {
        const float inv = 1.f / l;
        float4* dst = (float4*)(Oh + (int64_t)q_row * p.o_stride_n);
#pragma unroll
        for (int c = 0; c < D / 4; ++c)
            dst[c] = make_float4(o[4 * c] * inv, o[4 * c + 1] * inv, o[4 * c + 2] * inv, o[4 * c + 3] * inv);
    }
}

hipError_t launch_attn_f32(const AttnParams& p, int head_dim, bool dense, hipStream_t stream) {
    const dim3 grid(xcd_padded_blocks(p.total_tiles)), block(64);
    if (head_dim == 64) {
        if (dense) hipLaunchKernelGGL((attn_f32_kernel<64, true>), grid, block, 0, stream, p);
        else       hipLaunchKernelGGL((attn_f32_kernel<64, false>), grid, block, 0, stream, p);
    } else {
        if (dense) hipLaunchKernelGGL((attn_f32_kernel<128, true>), grid, block, 0, stream, p);
        else       hipLaunchKernelGGL((attn_f32_kernel<128, false>), grid, block, 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace grat
