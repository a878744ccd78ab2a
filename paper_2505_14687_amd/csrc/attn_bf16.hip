// bf16 block-sparse flash attention for gfx950 (grouped and dense), head_dim 128.
//
// Computes Sec. 3.1 Eq. 1 restricted to the attendable KV groups of Sec. 3.2.  Because all
// queries of a group share one KV list, every (query tile, KV tile) product is a full dense
// tile: no masking inside tiles, only a list walk around them.
//
// Work split: one workgroup = NWAVES wavefronts = 32*NWAVES queries of ONE group; each wave
// owns 32 queries.  K/V of the listed groups are gathered from row-major token order (rows of a
// group are runs of g_last contiguous tokens) into LDS in tiles of 64 tokens, double buffered.
//
// MFMA formulation (v_mfma_f32_32x32x16_bf16, 64-lane waves), "transposed" so that softmax
// statistics never cross lanes except once between the two halves of the wave:
//   S^T[key, query] = K_tile (A operand, rows = keys, from LDS) x Q^T (B operand, registers)
//       -> lane (query = lane % 32, half = lane / 32) holds 16 keys of that query per 32-key
//          block: key = 8*(r/4) + 4*half + r%4 for accumulator register r.
//   O^T[dim, query] += V^T_tile (A operand, rows = head dims, from LDS) x P^T (B operand)
//       -> P^T is exactly the S^T accumulator layout if the contraction index of the second
//          product is enumerated in that same (r, half) order; V^T is stored in LDS with its
//          token axis permuted to match, so P never leaves the lane's registers.
// Softmax runs in base 2 with scale*log2(e) folded into one FMA per score; running max, sum and
// the O accumulator stay fp32; P is rounded to bf16 (RNE) for the second product.
#include "grat_common.h"

namespace grat {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kD = 128;        // head_dim
constexpr int kBN = 64;        // KV tokens per LDS tile
constexpr int kKPitch = 136;   // bf16 per sK row (272 B: 16-lane b128 reads hit 64 distinct banks)
constexpr int kVPitch = 72;    // bf16 per sVt row (144 B)

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// max over the two lanes that hold the same query (lane and lane ^ 32)
__device__ __forceinline__ float max_across_halves(float x) {
    return fmaxf(x, __shfl_xor(x, 32));
}
__device__ __forceinline__ float sum_across_halves(float x) { return x + __shfl_xor(x, 32); }

template <int NWAVES, bool DENSE>
__global__ __launch_bounds__(NWAVES * 64, 2) void attn_bf16_kernel(AttnParams p) {
    constexpr int NT = NWAVES * 64;
    constexpr int BM = NWAVES * 32;
    // K tile chunks: 64 tokens x 16 chunks of 8 bf16.  V units: 16 token quads x 16 dim chunks.
    // With 512 threads the upper half of the block loads K and the lower half V; with fewer
    // threads everyone does both.
    constexpr bool SPLIT = NT == 512;
    constexpr int KT = SPLIT ? 256 : NT;          // threads loading K
    constexpr int VT = SPLIT ? 256 : NT;          // threads loading V
    constexpr int K_PER = 1024 / KT;              // 16-byte chunks per K-loading thread
    constexpr int V_PER = (256 + VT - 1) / VT;    // 4x8 units per V-loading thread

    __shared__ __attribute__((aligned(16))) uint16_t sK[2][kBN][kKPitch];
    __shared__ __attribute__((aligned(16))) uint16_t sVt[2][kD][kVPitch];
    extern __shared__ int32_t s_dyn[];   // [n_g] intra-group token offsets, then [max_kv] group origins

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int qcol = lane & 31;   // query within the wave's 32
    const int half = lane >> 5;

    const int tile = xcd_contiguous_tile(blockIdx.x, p.total_tiles);
    if (tile >= p.total_tiles) return;

    const Geometry& geo = p.geo;
    const int tiles_per_head = DENSE ? p.q_tiles : geo.num_groups * p.q_tiles;
    const int bh = tile / tiles_per_head;
    const int t_in_head = tile % tiles_per_head;
    const int64_t head_off = (int64_t)(bh / p.heads) * p.stride_b + (int64_t)(bh % p.heads) * p.stride_h;
    const uint16_t* Qh = (const uint16_t*)p.Q + head_off;
    const uint16_t* Kh = (const uint16_t*)p.K + head_off;
    const uint16_t* Vh = (const uint16_t*)p.V + head_off;
    uint16_t* Oh = (uint16_t*)p.O + head_off;
    const int stride_n = p.stride_n;

    int32_t* s_off = s_dyn;
    int32_t* s_origin = s_dyn + (DENSE ? 0 : geo.group_tokens);

    int n_iters;        // KV tiles to walk
    int tiles_per_group = 1;
    int q_row;          // token row of this lane's query
    bool q_valid = true;
    if (DENSE) {
        n_iters = (p.n_tokens + kBN - 1) / kBN;
        q_row = t_in_head * BM + wave * 32 + qcol;
        q_valid = q_row < p.n_tokens;
        if (!q_valid) q_row = p.n_tokens - 1;
    } else {
        const int gamma = t_in_head / p.q_tiles;
        const int qt = t_in_head % p.q_tiles;
        const int n_g = geo.group_tokens;
        const int T12 = geo.T[1] * geo.T[2], g12 = geo.g[1] * geo.g[2], G12 = geo.G[1] * geo.G[2];
        for (int t = tid; t < n_g; t += NT)
            s_off[t] = (t / g12) * T12 + ((t / geo.g[2]) % geo.g[1]) * geo.T[2] + t % geo.g[2];
        const int cnt = p.kv_count[gamma];
        for (int i = tid; i < cnt; i += NT) {
            const int gid = p.kv_index[(int64_t)gamma * p.max_kv + i];
            s_origin[i] = (gid / G12) * geo.g[0] * T12 + ((gid / geo.G[2]) % geo.G[1]) * geo.g[1] * geo.T[2] +
                          (gid % geo.G[2]) * geo.g[2];
        }
        __syncthreads();
        tiles_per_group = n_g / kBN;
        n_iters = cnt * tiles_per_group;
        const int q_origin = (gamma / G12) * geo.g[0] * T12 + ((gamma / geo.G[2]) % geo.G[1]) * geo.g[1] * geo.T[2] +
                             (gamma % geo.G[2]) * geo.g[2];
        q_row = q_origin + s_off[qt * BM + wave * 32 + qcol];
    }

    // Q^T fragments (B operand): this lane's query, dims 16*ks + 8*half .. +7
    bf16x8 qf[kD / 16];
    {
        const uint16_t* src = Qh + (uint32_t)q_row * stride_n + 8 * half;
#pragma unroll
        for (int ks = 0; ks < kD / 16; ++ks) qf[ks] = *(const bf16x8*)(src + 16 * ks);
    }

    f32x16 oacc[kD / 32];
#pragma unroll
    for (int db = 0; db < kD / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    float m_run = -INFINITY;   // running max of raw scores (before scale)
    float l_run = 0.f;         // this lane's share of the running sum (its 32 keys per tile)
    const float c = p.scale_log2;

    // ---- loader roles -------------------------------------------------------------------
    const bool loads_k = !SPLIT || tid >= 256;
    const bool loads_v = !SPLIT || tid < 256;
    const int ktid = SPLIT ? tid - 256 : tid;
    const int vtid = tid;
    uint4 kreg[K_PER];
    uint4 vreg[V_PER][4];

    // token row of token `kk` (0..63) of KV tile `it`
    auto kv_row = [&](int gi, int j, int it, int kk) -> int {
        if (DENSE) return min(it * kBN + kk, p.n_tokens - 1);
        return s_origin[gi] + s_off[j * kBN + kk];
    };
    auto issue_loads = [&](int gi, int j, int it) {
        if (loads_k) {
#pragma unroll
            for (int i = 0; i < K_PER; ++i) {
                const int ch = ktid + i * KT;
                const int row = kv_row(gi, j, it, ch >> 4);
                kreg[i] = *(const uint4*)(Kh + (uint32_t)row * stride_n + (ch & 15) * 8);
            }
        }
        if (loads_v) {
#pragma unroll
            for (int i = 0; i < V_PER; ++i) {
                const int u = vtid + i * VT;
                if (u < 256) {
                    const int kq = u >> 4, dc = u & 15;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int row = kv_row(gi, j, it, 4 * kq + e);
                        vreg[i][e] = *(const uint4*)(Vh + (uint32_t)row * stride_n + dc * 8);
                    }
                }
            }
        }
    };
    auto store_tiles = [&](int buf) {
        if (loads_k) {
#pragma unroll
            for (int i = 0; i < K_PER; ++i) {
                const int ch = ktid + i * KT;
                *(uint4*)&sK[buf][ch >> 4][(ch & 15) * 8] = kreg[i];
            }
        }
        if (loads_v) {
#pragma unroll
            for (int i = 0; i < V_PER; ++i) {
                const int u = vtid + i * VT;
                if (u < 256) {
                    const int kq = u >> 4, dc = u & 15;
                    // token quad kq lands at permuted quad position (swap its two low bits): the
                    // order in which the S^T accumulator enumerates keys
                    const int pos = 4 * ((kq & ~3) | ((kq & 1) << 1) | ((kq >> 1) & 1));
                    const uint32_t* w0 = (const uint32_t*)&vreg[i][0];
                    const uint32_t* w1 = (const uint32_t*)&vreg[i][1];
                    const uint32_t* w2 = (const uint32_t*)&vreg[i][2];
                    const uint32_t* w3 = (const uint32_t*)&vreg[i][3];
#pragma unroll
                    for (int dw = 0; dw < 4; ++dw) {
                        uint2 even, odd;   // dims 2*dw and 2*dw+1 of the chunk, 4 tokens each
                        even.x = (w0[dw] & 0xffffu) | (w1[dw] << 16);
                        even.y = (w2[dw] & 0xffffu) | (w3[dw] << 16);
                        odd.x = (w0[dw] >> 16) | (w1[dw] & 0xffff0000u);
                        odd.y = (w2[dw] >> 16) | (w3[dw] & 0xffff0000u);
                        *(uint2*)&sVt[buf][dc * 8 + 2 * dw][pos] = even;
                        *(uint2*)&sVt[buf][dc * 8 + 2 * dw + 1][pos] = odd;
                    }
                }
            }
        }
    };

    if (n_iters == 0) return;   // an empty list is outside the contract; never touch memory for it

    // ---- prologue ------------------------------------------------------------------------
    int gi_next = 0, j_next = 0;   // list entry / tile-in-group of the NEXT tile to load
    auto advance = [&]() {
        if (++j_next == tiles_per_group) { j_next = 0; ++gi_next; }
    };
    issue_loads(gi_next, j_next, 0);
    advance();
    store_tiles(0);
    __syncthreads();

    int buf = 0;
    for (int it = 0; it < n_iters; ++it) {
        const bool more = it + 1 < n_iters;
        if (more) {
            issue_loads(gi_next, j_next, it + 1);
            advance();
        }

        // ---- S^T = K_tile x Q^T: two 32-key blocks -------------------------------------
        f32x16 sacc[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[kb][r] = 0.f;
            const uint16_t* arow = &sK[buf][32 * kb + qcol][8 * half];
#pragma unroll
            for (int ks = 0; ks < kD / 16; ++ks) {
                const bf16x8 a = *(const bf16x8*)(arow + 16 * ks);
                sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], sacc[kb], 0, 0, 0);
            }
        }

        // dense tail: keys past the end of the sequence get weight 0
        if (DENSE && (it + 1) * kBN > p.n_tokens) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = it * kBN + 32 * kb + 8 * (r >> 2) + 4 * half + (r & 3);
                    if (key >= p.n_tokens) sacc[kb][r] = -INFINITY;
                }
        }

        // ---- online softmax (base 2) ------------------------------------------------------
        float mx = sacc[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kb][r]);
        mx = max_across_halves(mx);
        const float m_new = fmaxf(m_run, mx);
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);   // first tile: 0
        const float mc = m_new * c;
        m_run = m_new;
        float lsum = 0.f;
        uint32_t pw[2][8];   // P^T as bf16 pairs, in accumulator register order
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                const float p0 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][r], c, -mc));
                const float p1 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][r + 1], c, -mc));
                lsum += p0 + p1;
                pw[kb][r >> 1] = pack_bf16(p0, p1);
            }
        l_run = fmaf(l_run, alpha, lsum);
#pragma unroll
        for (int db = 0; db < kD / 32; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;

        // ---- O^T += V^T_tile x P^T: four 16-key steps x four 32-dim blocks -----------------
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const uint32_t* w = &pw[s >> 1][4 * (s & 1)];
            const uint4 braw = make_uint4(w[0], w[1], w[2], w[3]);
            const bf16x8 b = __builtin_bit_cast(bf16x8, braw);
#pragma unroll
            for (int db = 0; db < kD / 32; ++db) {
                const bf16x8 a = *(const bf16x8*)&sVt[buf][32 * db + qcol][16 * s + 8 * half];
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, oacc[db], 0, 0, 0);
            }
        }

        if (more) store_tiles(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }

    // ---- epilogue: normalise, round to bf16, store ------------------------------------------
    const float inv = 1.f / sum_across_halves(l_run);
    if (q_valid) {
        uint16_t* dst = Oh + (uint32_t)q_row * stride_n + 4 * half;
#pragma unroll
        for (int db = 0; db < kD / 32; ++db)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                uint2 v;
                v.x = pack_bf16(oacc[db][4 * rq] * inv, oacc[db][4 * rq + 1] * inv);
                v.y = pack_bf16(oacc[db][4 * rq + 2] * inv, oacc[db][4 * rq + 3] * inv);
                *(uint2*)(dst + 32 * db + 8 * rq) = v;
            }
    }
}

template <int NWAVES>
static hipError_t launch_one(const AttnParams& p, bool dense, hipStream_t stream) {
    const dim3 grid(xcd_padded_blocks(p.total_tiles)), block(NWAVES * 64);
    const size_t dyn = dense ? 0 : sizeof(int32_t) * ((size_t)p.geo.group_tokens + p.max_kv);
    if (dense) hipLaunchKernelGGL((attn_bf16_kernel<NWAVES, true>), grid, block, dyn, stream, p);
    else       hipLaunchKernelGGL((attn_bf16_kernel<NWAVES, false>), grid, block, dyn, stream, p);
    return hipGetLastError();
}

// p.q_tiles was computed by the host for the query-tile height chosen here: 256, 128 or 64 rows.
hipError_t launch_attn_bf16(const AttnParams& p, bool dense, hipStream_t stream) {
    const int bm = dense ? 256 : (p.geo.group_tokens / p.q_tiles);
    if (bm == 256) return launch_one<8>(p, dense, stream);
    if (bm == 128) return launch_one<4>(p, dense, stream);
    return launch_one<2>(p, dense, stream);
}

}  // namespace grat
