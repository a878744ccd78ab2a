// Block-sparse flash attention on the matrix cores of gfx950 (grouped, dense, joint), bf16 or half,
// head_dim 128 or 64.  The kernel template; its instantiations are compiled in attn_mfma_*.hip.
//
// Computes Sec. 3.1 Eq. 1 restricted to the attendable KV groups of Sec. 3.2.  Because all
// queries of a group share one KV list, every (query tile, KV tile) product is a full dense
// tile: no masking inside tiles, only a list walk around them.
//
// Work split: one workgroup = NWAVES wavefronts = 32*NWAVES queries of ONE group; each wave
// owns 32 queries.  K/V of the listed groups are gathered from row-major token order (a group's
// rows are runs of g_last contiguous tokens) straight into LDS with global_load_lds_dwordx4,
// in tiles of 64 tokens, double buffered; no registers are staged and nothing is permuted in
// HBM.
//
// MFMA formulation (v_mfma_f32_32x32x16_bf16, 64-lane waves), "transposed" so that softmax
// statistics never cross lanes except once between the two halves of the wave:
//   S^T[key, query] = K_tile (A operand, rows = keys, from LDS) x Q^T (B operand, registers)
//       -> lane (query = lane % 32, half = lane / 32) holds 16 keys of that query per 32-key
//          block: key = 8*(r/4) + 4*half + r%4 for accumulator register r.
//   O^T[dim, query] += V^T_tile (A operand, rows = head dims) x P^T (B operand)
//       -> P^T is exactly the S^T accumulator layout if the contraction index of the second
//          product is enumerated in that same (r, half) order, so P never leaves the lane's
//          registers; the matching V^T fragments come out of the row-major V tile through the
//          LDS transpose read ds_read_b64_tr_b16.
// Softmax runs in base 2 with scale*log2(e) folded into one FMA per score; the reference
// maximum, the running sum and the O accumulator stay fp32; P is rounded to bf16 (RNE) for the
// second product; the row sum is taken over the unrounded fp32 weights with plain adds.
//
// Schedule: one barrier per KV tile, and between two barriers ONE instruction stream per wave in
// which the work is software-pipelined by 32-key blocks (half a tile): while the matrix pipe forms
// the scores of block h, the vector ALU turns the scores of block h-1 into weights and the matrix
// pipe adds block h-2 to O.  The three stages of a half step do not depend on each other, so every
// MFMA is followed by its share of the vector work: a 32x32x16 MFMA holds the matrix pipe for 32
// cycles but the issue port for 8, and 24 cycles of other vector instructions fit behind it.
// (Measured on this chip: v_dot2c_f32_bf16 is not among them - it waits for the matrix pipe and
// holds it for 16 cycles - which is why the row sum uses v_add_f32.)
#pragma once
#include <type_traits>

#include "grat_common.h"

namespace grat {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(8))) short frag8;   // 8 sixteen-bit elements of either type
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#define LDS_PTR(T) __attribute__((address_space(3))) T*

constexpr int kD = 128;               // head_dim
constexpr int kRowBytes = kD * 2;     // 256 B per token row
// KV tokens per LDS tile (template argument BN of the kernel): 64, or 32 as an option for the 2-wave
// workgroups (64 queries) of small groups, whose four tiles then take 32 KiB so that four workgroups
// (two waves per SIMD) share a compute unit instead of two - worth it for short lists, where a
// workgroup's fixed cost weighs most; long lists run better on 64-key tiles (half as many barriers,
// tile look-ups and load instructions per key).
constexpr int kFragAhead = 2;         // an MFMA's LDS fragment is read this many MFMAs ahead of it

// LDS tiles are unpadded [64 rows][16 chunks of 16 B]; the chunk index is XOR-swizzled per row so
// that the fragment reads are bank-conflict free.  K is read with ds_read_b128 by lanes holding
// consecutive rows: spread rows over all 16 chunk positions (and keep the two dim-halves of a
// row apart).  V is read with the 8-byte transpose read by 4 rows x 4 chunks at a time: move
// each of 4 consecutive rows to a different group of 4 chunks.
__device__ __forceinline__ int k_swizzle(int row) { return ((row & 7) << 1) | ((row >> 3) & 1); }
__device__ __forceinline__ int v_swizzle(int row) { return (row & 3) << 2; }

// What depends on the 16-bit element type (F16 = false: bfloat16, true: IEEE half).  Fragments
// travel as type-neutral frag8 and are reinterpreted at the MFMA.
template <bool F16>
struct Elem {
    // a lane's block row sum (16 weights) beyond this forces a new reference maximum: every single
    // weight then stays inside the type's range (half: 65504) with its full relative precision
    static constexpr float kSumLimit = F16 ? 0x1p+15f : 0x1p+40f;
    static __device__ __forceinline__ f32x16 mfma(frag8 a, frag8 b, f32x16 c) {
        if constexpr (F16)
            return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
        else
            return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
    // two fp32 values rounded to nearest-even and packed (lo in the low half)
    static __device__ __forceinline__ uint32_t pack(float lo, float hi) {
        const f32x2 v = {lo, hi};
        if constexpr (F16) return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
        else return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    }
};

// Exchange between the two lanes that hold the same query (lane and lane ^ 32) with one
// v_permlane32_swap.  The two results are copied to scalars before they are reinterpreted:
// a bit cast applied directly to a vector element reads element 0 with this compiler.
__device__ __forceinline__ void swap_halves(float x, float& lower, float& upper) {
    const uint32_t a = __builtin_bit_cast(uint32_t, x);
    const auto r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
    const uint32_t r0 = r[0], r1 = r[1];
    lower = __builtin_bit_cast(float, r0);   // value held by the lane with the same query, half 0
    upper = __builtin_bit_cast(float, r1);   // ... half 1
}
__device__ __forceinline__ float max_across_halves(float x) {
    float lo, hi;
    swap_halves(x, lo, hi);
    return fmaxf(lo, hi);
}
__device__ __forceinline__ float sum_across_halves(float x) {
    float lo, hi;
    swap_halves(x, lo, hi);
    return lo + hi;
}

// (MODE: see AttnMode in grat_common.h)

// Box coordinates of an intra-group token, packed for the border tests of kRagged: 12 + 10 + 10 bits.
__device__ __forceinline__ uint32_t pack_coord(int c0, int c1, int c2) {
    return (uint32_t)c0 << 20 | (uint32_t)c1 << 10 | (uint32_t)c2;
}
// every coordinate of c at most the matching one of lim (lim = largest coordinates inside the grid)
__device__ __forceinline__ bool coord_inside(uint32_t c, uint32_t lim) {
    return (c >> 20) <= (lim >> 20) && ((c >> 10) & 1023u) <= ((lim >> 10) & 1023u) && (c & 1023u) <= (lim & 1023u);
}

// D = head_dim of the tensors, 128 or 64.  The LDS layout is 128 wide (kD) either way: for D = 64
// the tiles keep their 256-byte rows, same swizzles, same fragment addresses; the direct loads
// only fill the 8 chunk positions of every row that belong to real head dims (lanes whose
// position would hold a chunk that does not exist are masked off), the QK product contracts over
// the 4 fragments that exist, and the upper half of O^T is never formed, so no MFMA or LDS read is
// spent on padding (the unused chunk positions are never written and never read).
//
// One query tile: tile t_in_head of its kind in (batch, head) bh.  DENSE: it is a tile of consecutive
// query rows that walks the whole sequence (always in kDense, the prompt rows in kJoint), else a
// tile of one query group.  sK / sV: the workgroup's two K and two V tile buffers in LDS.
template <int NWAVES, int BN, int MODE, bool F16, int D, bool DENSE>
__device__ __forceinline__ void attn_tile(const AttnParams& p, const int bh, const int t_in_head,
                                          uint8_t (*sK)[BN * kRowBytes], uint8_t (*sV)[BN * kRowBytes],
                                          const int gamma_fixed = -1) {
    static_assert(BN == 64 || (BN == 32 && NWAVES == 2), "64-key tiles, or 32-key tiles for 2-wave workgroups");
    constexpr int kBN = BN;
    constexpr int kTileBytes = kBN * kRowBytes;
    static_assert(D == 128 || D == 64, "head_dim 128 or 64");
    using E = Elem<F16>;
    constexpr int NT = NWAVES * 64;
    constexpr int BM = NWAVES * 32;
    constexpr int LPW = kBN / (4 * NWAVES);   // 1-KiB direct loads (4 token rows) per wave per tile
    constexpr bool dense = DENSE;

    extern __shared__ int32_t s_dyn[];   // [n_g] row offsets inside a group, then [max_kv] group origins (kRagged: and the two tables below)
    constexpr bool kLists = MODE == kGrouped || MODE == kRagged;   // every KV tile comes from a listed group
    constexpr bool kLeadThenLists = MODE == kJoint && !DENSE;      // prompt tiles first, then the listed groups

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int qcol = lane & 31;   // query within the wave's 32
    const int half = lane >> 5;

    const Geometry& geo = p.geo;
    // (index decompositions go through host-prepared multipliers: see fastdiv.h)
    const int b_idx = (int)fdiv((uint32_t)bh, p.fd_heads), h_idx = bh - b_idx * p.heads;
    const int64_t head_off = (int64_t)b_idx * p.stride_b + (int64_t)h_idx * p.stride_h;
    const uint16_t* Qh = (const uint16_t*)p.Q + head_off;
    const uint16_t* Kh = (const uint16_t*)p.K + head_off;
    const uint16_t* Vh = (const uint16_t*)p.V + head_off;
    uint16_t* Oh = (uint16_t*)p.O + (int64_t)b_idx * p.o_stride_b + (int64_t)h_idx * p.o_stride_h;
    const int stride_n = p.stride_n;

    // s_rowbytes[t]: byte offset (row * stride_n * 2) of intra-group token t relative to its group's
    // first token - a group spans less than 4 GiB; s_origin[i]: ROW of the first token of the i-th
    // listed KV group - wave-uniform, turned into a 64-bit address in scalar registers, so the
    // sequence itself may be as large as memory (packed [B][N][3][H][d] layouts of long sequences)
    uint32_t* s_rowbytes = (uint32_t*)s_dyn;
    // kRagged: s_coord[t] = box coordinates of intra-group token t (behind s_rowbytes, so that it
    // stays 16-byte aligned), s_limit[i] = largest box coordinates of listed group i that are still
    // inside the grid (both packed)
    uint32_t* s_coord = s_rowbytes + geo.group_tokens;
    uint32_t* s_origin = (uint32_t*)s_dyn + (MODE == kDense ? 0 : (MODE == kRagged ? 2 : 1) * geo.group_tokens);
    uint32_t* s_limit = s_origin + p.max_kv;
    uint32_t q_limit = 0;   // kRagged: the same limit for the query group
    const uint32_t row_pitch = (uint32_t)stride_n * 2u;   // bytes between consecutive tokens

    int n_tiles;        // KV tiles to walk
    int tiles_per_group = 1;
    int n_listed = 1;   // grouped tiles: entries in s_origin
    int n_lead = 0;     // grouped tile of a joint sequence: leading KV tiles that hold the prompt tokens
    int mask_tile = -1, mask_valid = kBN;   // the one KV tile with fewer than kBN valid keys, if any
    // query rows of this wave: row i of its 32 is row q_first + i of the dense rows, resp. token
    // q_first + i of its group, whose first token is row q_base of the head
    uint32_t q_base = 0;
    int q_first;
    frag8 qf[kD / 16];   // Q^T fragments (B operand): this lane's query, dims 16*ks + 8*half .. +7
    if (dense) {
        n_tiles = (p.n_tokens + kBN - 1) / kBN;
        if (p.n_tokens % kBN) { mask_tile = n_tiles - 1; mask_valid = p.n_tokens % kBN; }
        q_first = t_in_head * BM + wave * 32;
    } else {
        int qt, gamma;
        if (gamma_fixed >= 0) {   // the caller has picked the group: t_in_head is the tile inside it
            gamma = gamma_fixed;
            qt = t_in_head;
        } else {
            const uint32_t u_group = fdiv((uint32_t)t_in_head, p.fd_q_tiles);
            qt = t_in_head - (int)u_group * p.q_tiles;
            gamma = strip_order_group_fast(u_group, geo.G[0] * geo.G[1], geo.G[2], p);
        }
        const int n_g = geo.group_tokens;
        const int T12 = geo.T[1] * geo.T[2];
        // row of the first token of group gid, relative to the first grid row
        auto group_origin = [&](uint32_t gid, int& p0, int& p1, int& p2) {
            uint32_t v, r2, q0, r1;
            fdivmod(gid, p.fd_G2, v, r2);
            fdivmod(v, p.fd_G1, q0, r1);
            p0 = (int)q0; p1 = (int)r1; p2 = (int)r2;
            return p0 * geo.g[0] * T12 + p1 * geo.g[1] * geo.T[2] + p2 * geo.g[2];
        };
        // box coordinates of token t of a group
        auto token_coord = [&](uint32_t t, int& c0, int& c1, int& c2) {
            uint32_t v, r2, q0, r1;
            fdivmod(t, p.fd_g2, v, r2);
            fdivmod(v, p.fd_g1, q0, r1);
            c0 = (int)q0; c1 = (int)r1; c2 = (int)r2;
        };
        const uint32_t grid_base = MODE == kJoint ? (uint32_t)p.grid_row0 : 0u;   // first grid row
        auto box_limit = [&](int gid) {   // largest box coordinates of group gid inside the grid
            int p0, p1, p2;
            group_origin((uint32_t)gid, p0, p1, p2);
            return pack_coord(min(geo.g[0], geo.T[0] - p0 * geo.g[0]) - 1, min(geo.g[1], geo.T[1] - p1 * geo.g[1]) - 1,
                              min(geo.g[2], geo.T[2] - p2 * geo.g[2]) - 1);
        };
        // The queries are asked for first of all, with their row offset worked out in arithmetic
        // rather than read from the table below: they come from HBM (nobody has touched them
        // before) and everything up to the first barrier then happens in the shadow of that fetch.
        {
            int gp0, gp1, gp2;
            const int q_origin = group_origin((uint32_t)gamma, gp0, gp1, gp2);
            q_base = grid_base + (uint32_t)q_origin;
            q_first = qt * BM + wave * 32;
            int c0, c1, c2;
            token_coord((uint32_t)(q_first + qcol), c0, c1, c2);
            uint32_t off = (uint32_t)(c0 * T12 + c1 * geo.T[2] + c2) * row_pitch;
            if (MODE == kRagged) {
                q_limit = box_limit(gamma);
                if (!coord_inside(pack_coord(c0, c1, c2), q_limit)) off = 0;   // a query outside the grid: any valid row will do
            }
            const uint8_t* src = (const uint8_t*)Qh + (uint64_t)q_base * row_pitch + off + 16 * half;
#pragma unroll
            for (int ks = 0; ks < kD / 16; ++ks) qf[ks] = ks < D / 16 ? *(const frag8*)(src + 32 * ks) : frag8{0, 0, 0, 0, 0, 0, 0, 0};
        }
        for (int t = tid; t < n_g; t += NT) {
            int c0, c1, c2;
            token_coord((uint32_t)t, c0, c1, c2);
            s_rowbytes[t] = (uint32_t)(c0 * T12 + c1 * geo.T[2] + c2) * row_pitch;
            if (MODE == kRagged) s_coord[t] = pack_coord(c0, c1, c2);
        }
        // (a caller-made list is taken as it is, but its count and entries are forced into range: a
        // bad list then gives wrong numbers, never an access outside the tables or the tensors)
        const int cnt = min(max(p.kv_count[gamma], 0), p.max_kv);
        for (int i = tid; i < cnt; i += NT) {
            const int gid = min(max(p.kv_index[(int64_t)gamma * p.max_kv + i], 0), geo.num_groups - 1);
            int p0, p1, p2;
            s_origin[i] = grid_base + (uint32_t)group_origin((uint32_t)gid, p0, p1, p2);
            if (MODE == kRagged) s_limit[i] = box_limit(gid);
        }
        __syncthreads();
        tiles_per_group = n_g / kBN;
        if (MODE == kJoint) {
            n_lead = (p.n_global + kBN - 1) / kBN;
            if (p.n_global % kBN) { mask_tile = n_lead - 1; mask_valid = p.n_global % kBN; }
        }
        n_tiles = n_lead + cnt * tiles_per_group;
        n_listed = cnt;
    }
    if (n_tiles == 0) return;   // an empty list is outside the contract; never touch memory for it
    // byte offset inside the head of row i of this wave's 32 query (= output) rows; the rows of a
    // dense tile past the last query re-read the last one and are never stored
    auto q_row_off = [&](int i) -> uint64_t {
        if (dense) return (uint64_t)(uint32_t)(p.dense_row0 + min(q_first + i, p.n_dense_rows - 1)) * row_pitch;
        return (uint64_t)q_base * row_pitch + s_rowbytes[q_first + i];
    };

    if (dense) {
        const uint8_t* src = (const uint8_t*)Qh + q_row_off(qcol) + 16 * half;
#pragma unroll
        for (int ks = 0; ks < kD / 16; ++ks) qf[ks] = ks < D / 16 ? *(const frag8*)(src + 32 * ks) : frag8{0, 0, 0, 0, 0, 0, 0, 0};
    }

    f32x16 oacc[D / 32];                  // O^T accumulator: blocks of 32 head dims
    f32x16 S[2];                          // S^T of the two 32-key blocks in flight
    uint32_t pw[2][8];                    // their weights P^T as 16-bit pairs, in accumulator order
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) S[kb][r] = 0.f;
#pragma unroll
        for (int r = 0; r < 8; ++r) pw[kb][r] = 0u;
    }
    float m_ref = -INFINITY;   // reference maximum of raw scores the weights are taken against
    float l_run = 0.f;         // this lane's share of the running sum (its 16 keys per block)
    const float c = p.scale_log2;

    // ---- tile loads: LPW one-KiB pieces per wave; lane -> (row = 4*piece + lane/16, chunk) ----
    // Address of a piece = head base + (wave-uniform) byte offset of the tile's first token, kept
    // in scalar registers, + a per-lane byte offset: row within the group (one table read) plus
    // the swizzled 16-byte chunk of the row.
    int load_row[LPW];
    uint32_t load_kcol[LPW], load_vcol[LPW];
    bool k_on[LPW], v_on[LPW];
#pragma unroll
    for (int k = 0; k < LPW; ++k) {
        const int row = 4 * (wave * LPW + k) + (lane >> 4);
        load_row[k] = row;
        load_kcol[k] = (uint32_t)(((lane & 15) ^ k_swizzle(row)) * 16);   // byte offset of the global chunk
        load_vcol[k] = (uint32_t)(((lane & 15) ^ v_swizzle(row)) * 16);
        k_on[k] = load_kcol[k] < (uint32_t)D * 2;   // D = 64: this lane's LDS position holds a real chunk
        v_on[k] = load_vcol[k] < (uint32_t)D * 2;
    }
    struct TileAddr {
        uint32_t base;        // wave-uniform
        uint32_t off[LPW];    // per lane
    };
    int gi_k = 0, j_k = 0, gi_v = 0, j_v = 0;   // list entry / tile-in-group of the next K (dense walk: and V) tile
    TileAddr ka, va;
    // V(t) lies in the rows of K(t): where the rows come out of table reads, its address is taken
    // from K's with the other swizzle in the column part instead of being looked up again (+0.7 %;
    // the dense walk, whose addresses are arithmetic, measured 1 % slower that way and forms both)
    uint32_t k_to_vcol[LPW];
#pragma unroll
    for (int k = 0; k < LPW; ++k) k_to_vcol[k] = load_vcol[k] - load_kcol[k];
    auto v_from_k = [&](TileAddr& v, const TileAddr& kk) {
        v.base = kk.base;
#pragma unroll
        for (int k = 0; k < LPW; ++k) v.off[k] = kk.off[k] + k_to_vcol[k];
    };
    // Offsets of a tile are looked up one tile before it is fetched, so the table reads never sit
    // between a barrier and the loads that follow it.
    auto tile_addr = [&](TileAddr& a, const uint32_t* col, int t, int& gi, int& j) {
        if (dense) {
            // consecutive rows of the whole sequence; rows past the end re-read the last token (masked later)
            a.base = (uint32_t)(t * kBN);
#pragma unroll
            for (int k = 0; k < LPW; ++k)   // (also asked for tiles past the end, never fetched: keep the offset small)
                a.off[k] = (uint32_t)max(0, min(load_row[k], p.n_tokens - 1 - t * kBN)) * row_pitch + col[k];
        } else if (kLeadThenLists) {
            // Both kinds of address are formed every time and one is selected, so that there is no
            // branch (and no block of table reads with waits of its own) inside a step.
            const bool lead = t < n_lead;
            const uint32_t base_list = __builtin_amdgcn_readfirstlane(s_origin[min(gi, n_listed - 1)]);
            a.base = lead ? (uint32_t)(p.global_row0 + t * kBN) : base_list;
#pragma unroll
            for (int k = 0; k < LPW; ++k) {
                const uint32_t o_list = s_rowbytes[j * kBN + load_row[k]];
                const uint32_t o_lead = (uint32_t)max(0, min(load_row[k], p.n_global - 1 - t * kBN)) * row_pitch;
                a.off[k] = (lead ? o_lead : o_list) + col[k];
            }
            if (!lead && ++j == tiles_per_group) { j = 0; ++gi; }
        } else {
            a.base = __builtin_amdgcn_readfirstlane(s_origin[min(gi, n_listed - 1)]);   // (may be asked past the end)
            // kRagged: rows of the box beyond the last token of the sequence are pulled back onto it
            const uint64_t to_end = (uint64_t)((uint32_t)geo.n_tokens - 1u - a.base) * row_pitch;
            const uint32_t max_off = to_end > 0xffffffffull ? 0xffffffffu : (uint32_t)to_end;
#pragma unroll
            for (int k = 0; k < LPW; ++k) {
                const uint32_t o = s_rowbytes[j * kBN + load_row[k]];
                a.off[k] = (MODE == kRagged ? min(o, max_off) : o) + col[k];
            }
            if (++j == tiles_per_group) { j = 0; ++gi; }
        }
    };
    // The loads are written as inline assembly on purpose: the compiler's wait-count pass treats a
    // direct-to-LDS load it can see as a possible alias of every later LDS read and would drain
    // the prefetch before the first fragment read that follows.  Completion is waited for
    // explicitly (s_waitcnt vmcnt(0)) before the barrier that publishes the tile.
    auto issue_tile = [&](const uint16_t* head, uint8_t* dst_tile, const TileAddr& a, const bool (&on)[LPW]) {
        // (made uniform again here: carried across iterations the offset may sit in a vector register)
        const uint8_t* base = (const uint8_t*)head + (uint64_t)__builtin_amdgcn_readfirstlane(a.base) * row_pitch;
#pragma unroll
        for (int k = 0; k < LPW; ++k) {
            // LDS destination of this wave's piece; the hardware adds lane * 16
            const uint32_t lds_dst = __builtin_amdgcn_readfirstlane(
                (uint32_t)(uintptr_t)(LDS_PTR(uint8_t))(dst_tile + (wave * LPW + k) * 1024));
            // (one wait state between the M0 write and the LDS-DMA instruction that reads it)
            if (D == 128 || on[k])
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                             :: "s"(lds_dst), "v"(a.off[k]), "s"(base) : "memory", "m0");
        }
    };

    // ---- fragment addresses ----------------------------------------------------------------
    // K (A operand of S^T): row 32*kb + qcol, chunk (2*ks + half) ^ swizzle(row)
    const int k_lane_base = qcol * kRowBytes;
    const int k_x = k_swizzle(qcol) ^ half;          // (2*ks + half) ^ sw == (2*ks) ^ (sw ^ half)
    // V (A operand of O^T) via transpose reads: 16-lane block -> (e = row in quad, cq = 4-dim column)
    const int tr_e = (lane & 15) >> 2, tr_cq = lane & 3, tr_dsel = (lane >> 4) & 1;
    const int v_lane_base = (4 * half + tr_e) * kRowBytes + 8 * (tr_cq & 1);
    // chunk = 4*db + 2*dsel + cq/2, swizzled with 4*(row & 3) = 4*e  ->  4*(db ^ e) + 2*dsel + cq/2
    const int v_chunk_lo = 2 * tr_dsel + (tr_cq >> 1);

    // ---- the software pipeline ---------------------------------------------------------------
    // Work is cut into 32-key blocks (half a K/V tile).  For block h the three stages run one half
    // step apart:  QK(h) -> S[h % 2]   |   weights(h-1): S[(h-1) % 2] -> pw[(h-1) % 2]   |
    // PV(h-2) with pw[h % 2].  Inside a half step the three streams are independent of each other,
    // so the vector work can be dealt out evenly between the MFMAs: a 32x32x16 MFMA occupies the
    // matrix pipe for 32 cycles but the issue port for only 8, and up to 24 cycles of other vector
    // instructions fit in its shadow.  (The packed dot product is not one of them: it runs on the
    // matrix pipe and waits for it, so the row sum is taken with plain adds.)
    // (the per-lane part of the K fragment addresses is formed once and pinned in registers: left to
    // itself the compiler re-adds the swizzled chunk offset in front of every read)
    uint32_t k_addr[D / 16];
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
        k_addr[ks] = (uint32_t)(uintptr_t)(LDS_PTR(uint8_t))(&sK[0][0] + k_lane_base + (((2 * ks) ^ k_x) << 4));
        asm volatile("" : "+v"(k_addr[ks]));
    }
    auto k_frag = [&](int kbuf, int kb, int ks) -> frag8 {
        return *(LDS_PTR(const frag8))(uintptr_t)(k_addr[ks] + kbuf * kTileBytes + (kBN == 64 ? kb * 32 * kRowBytes : 0));
    };
    auto v_frag = [&](int vbuf, int kb, int s2, int db) -> frag8 {
        const uint8_t* src = sV[vbuf] + v_lane_base + ((kBN == 64 ? 32 * kb : 0) + 16 * s2) * kRowBytes + ((4 * (db ^ tr_e) + v_chunk_lo) << 4);
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))src);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(src + 8 * kRowBytes));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    auto mask_tail = [&](int kb) {   // the ragged tile: keys past the end of their run get weight 0
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = (kBN == 64 ? 32 * kb : 0) + 8 * (r >> 2) + 4 * half + (r & 3);
            if (key >= mask_valid) S[kb][r] = -INFINITY;
        }
    };
    // kRagged: called once per 32-key block, in walk order.  Keys of a border group's box that lie
    // outside the grid get weight 0.  (The first block of every box holds its first token, which is
    // always inside, so the first block of a walk never ends up without a finite score.)
    int gi_m = 0, j_m = 0;   // list entry / tile-in-group of the tile whose scores are being weighted
    const uint32_t full_box = pack_coord(geo.g[0] - 1, geo.g[1] - 1, geo.g[2] - 1);
    auto mask_outside = [&](int kb) {
        const uint32_t lim = __builtin_amdgcn_readfirstlane(s_limit[min(gi_m, n_listed - 1)]);
        if (lim != full_box) {
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                // accumulator registers 4*rq .. 4*rq+3 hold 4 consecutive keys
                const uint4 cc = *(const uint4*)&s_coord[j_m * kBN + (kBN == 64 ? 32 * kb : 0) + 8 * rq + 4 * half];
                if (!coord_inside(cc.x, lim)) S[kb][4 * rq] = -INFINITY;
                if (!coord_inside(cc.y, lim)) S[kb][4 * rq + 1] = -INFINITY;
                if (!coord_inside(cc.z, lim)) S[kb][4 * rq + 2] = -INFINITY;
                if (!coord_inside(cc.w, lim)) S[kb][4 * rq + 3] = -INFINITY;
            }
        }
        if ((kBN == 32 || kb == 1) && ++j_m == tiles_per_group) { j_m = 0; ++gi_m; }
    };
    // Weights are taken against a reference maximum m_ref that is only as fresh as it needs to be:
    // the common path computes exp2(c*s - c*m_ref) without looking at the block's own maximum and
    // checks afterwards that no row sum of the block left the safe range.  Only then (and on the
    // first block, whose maximum is taken up front) is the true maximum computed, O and the running
    // sum rescaled, and the block's weights recomputed.  Any reference gives the same quotient
    // O / l; this one keeps every weight below 2^40, which bf16 and the fp32 accumulators hold
    // without loss of relative accuracy.
    auto block_max = [&](int kb) {
        float mx = S[kb][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, S[kb][r]);
        return max_across_halves(mx);
    };
    auto refresh_reference = [&](int kb, float& ls) {   // the rare path
        const float m_new = fmaxf(m_ref, block_max(kb));
        const float alpha = __builtin_amdgcn_exp2f((m_ref - m_new) * c);
        m_ref = m_new;
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
        const float mc = m_ref * c;
        ls = 0.f;
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            const float p0 = __builtin_amdgcn_exp2f(fmaf(S[kb][r], c, -mc));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(S[kb][r + 1], c, -mc));
            pw[kb][r >> 1] = E::pack(p0, p1);
            ls += p0 + p1;
        }
    };

    // ---- prologue: K tile 0 -----------------------------------------------------------------
    tile_addr(ka, load_kcol, 0, gi_k, j_k);
    issue_tile(Kh, sK[0], ka, k_on);
    if (dense) tile_addr(va, load_vcol, 0, gi_v, j_v);
    else v_from_k(va, ka);
    if (1 < n_tiles) tile_addr(ka, load_kcol, 1, gi_k, j_k);

    // swap_barrier(t) publishes K(t) and V(t-1), fetched during the previous tile, and frees the
    // buffers of K(t-1) and V(t-2), which are refilled with K(t+1) and V(t) right away.
    // next_addrs(t): looks up where K(t+2) and V(t+1) lie (one tile before they are fetched, so that
    // the table reads never sit between a barrier and the loads that follow it).
    // 32-key tiles (2-wave workgroups): a step is a single 32-key block, so PV trails QK by two tiles
    // and V(t) is only fetched at barrier t+1, into the buffer V(t-2) was read from during step t;
    // vb = where V(t-1) lies, one tile behind va.
    TileAddr vb = va;
    auto next_addrs = [&](int t) {
        // (looked up unconditionally, also past the last tile, so that the table reads stay inside the
        // straight-line block around them instead of becoming a block of their own with its own waits)
        if (kBN == 32) vb = va;
        if (dense) tile_addr(va, load_vcol, t + 1, gi_v, j_v);
        else v_from_k(va, ka);   // tile t + 1, whose K part has just been asked for
        tile_addr(ka, load_kcol, t + 2, gi_k, j_k);
    };
    auto swap_barrier = [&](int t) {
        __builtin_amdgcn_s_waitcnt(0);   // this wave's direct-to-LDS loads have landed
        __syncthreads();                 // ... everyone's have, and all reads of the buffers to refill are done
        if (t + 1 < n_tiles) issue_tile(Kh, sK[(t + 1) & 1], ka, k_on);
        if (kBN == 64) {
            if (t < n_tiles) issue_tile(Vh, sV[t & 1], va, v_on);
        } else {
            if (t >= 1 && t - 1 < n_tiles) issue_tile(Vh, sV[(t - 1) & 1], vb, v_on);
        }
    };

    // One step = the two half steps between two barriers, as one instruction stream.  Half KB (0, 1)
    // works on keys 32*KB .. 32*KB+31 of its tiles.  Per half, QK: form S[KB] from the K tile in
    // sK[kbuf]; SM: weights of the block whose scores are in S[KB ^ 1] (0 none, 1 against the current
    // reference, 2 first block of the walk: the reference is its maximum); PV: O^T += V^T P^T for
    // half KB of the V tile in sV[vbuf], with the weights in pw[KB].  check: the walk contains a tile
    // with fewer than 64 valid keys; t_sm0 / t_sm1 = tile index of the block weighted in each half.
    // The items (one MFMA each, with its fragment read kFragAhead items ahead) run in one rolling
    // sequence over both halves; the vector chunks of a half are dealt out over its items.
    auto step = [&](auto qk0_c, auto sm0_c, auto pv0_c, auto qk1_c, auto sm1_c, auto pv1_c, auto check, auto kbuf_c,
                    int vbuf, int t_sm0, int t_sm1) {
        constexpr int kbuf = decltype(kbuf_c)::value;
        constexpr int SMm[2] = {decltype(sm0_c)::value, decltype(sm1_c)::value};
        constexpr int NQ[2] = {decltype(qk0_c)::value ? D / 16 : 0, decltype(qk1_c)::value ? D / 16 : 0};
        constexpr int NP[2] = {decltype(pv0_c)::value ? 2 * (D / 32) : 0, decltype(pv1_c)::value ? 2 * (D / 32) : 0};
        constexpr int NI[2] = {NQ[0] + NP[0], NQ[1] + NP[1]};
        constexpr int NT = NI[0] + NI[1], AHEAD = kFragAhead;
        frag8 fr[NT > 0 ? NT : 1];
        auto fetch = [&](int i) {
            const int h = i < NI[0] ? 0 : 1, j = i - (h ? NI[0] : 0);
            if (j < NQ[h]) fr[i] = k_frag(kbuf, h, j);
            else fr[i] = v_frag(vbuf, h, (j - NQ[h]) / (D / 32), (j - NQ[h]) % (D / 32));
        };
        float mc = 0.f, ls0 = 0.f, ls1 = 0.f, t1[8], e0[8];
        auto sm_begin = [&](int h) {   // h: the half; the block being weighted is h ^ 1
            if (SMm[h] == 0) return;
            const int sb = h ^ 1;
            if constexpr (decltype(check)::value) {
                if ((h ? t_sm1 : t_sm0) == mask_tile) mask_tail(sb);
            }
            if (MODE == kRagged) mask_outside(sb);
            if (SMm[h] == 2) m_ref = block_max(sb);
            mc = m_ref * c;
        };
        // two vector chunks per pair of scores: {fma, fma, exp2} and {exp2, pack, add, add}
        auto sm_chunk = [&](int h, int ch) {
            const int g = ch >> 1, sb = h ^ 1;
            if ((ch & 1) == 0) {
                const float t0 = fmaf(S[sb][2 * g], c, -mc);
                t1[g] = fmaf(S[sb][2 * g + 1], c, -mc);
                e0[g] = __builtin_amdgcn_exp2f(t0);
            } else {
                const float e1 = __builtin_amdgcn_exp2f(t1[g]);
                pw[sb][g] = E::pack(e0[g], e1);
                asm volatile("" : "+v"(pw[sb][g]));   // (keeps the conversion here: its first use is a block later)
                ls0 = g == 0 ? e0[g] : ls0 + e0[g];
                ls1 = g == 0 ? e1 : ls1 + e1;
            }
        };
        auto sm_end = [&](int h) {
            if (SMm[h] == 0) return;
            float ls = ls0 + ls1;
            if (SMm[h] == 1) {
                if (__builtin_amdgcn_ballot_w64(!(ls < E::kSumLimit)) != 0) refresh_reference(h ^ 1, ls);
            }
            l_run += ls;
        };
        // first of the 16 chunks of half h that go with its item j
        auto chunk_lo = [&](int h, int j) { return SMm[h] ? j * 16 / NI[h] : 0; };
#pragma unroll
        for (int a = 0; a < AHEAD && a < NT; ++a) fetch(a);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            sm_begin(h);
            if (NI[h] == 0) {
#pragma unroll
                for (int ch = 0; ch < (SMm[h] ? 16 : 0); ++ch) sm_chunk(h, ch);
            }
#pragma unroll
            for (int j = 0; j < NI[h]; ++j) {
                const int i = (h ? NI[0] : 0) + j;
                if (i + AHEAD < NT) fetch(i + AHEAD);
                if (j < NQ[h]) {
                    if (j == 0) {
                        f32x16 zero;
#pragma unroll
                        for (int r = 0; r < 16; ++r) zero[r] = 0.f;
                        S[h] = E::mfma(fr[i], qf[j], zero);
                    } else {
                        S[h] = E::mfma(fr[i], qf[j], S[h]);
                    }
                } else {
                    const int s2 = (j - NQ[h]) / (D / 32), db = (j - NQ[h]) % (D / 32);
                    const uint32_t* w = &pw[h][4 * s2];
                    const frag8 b = __builtin_bit_cast(frag8, make_uint4(w[0], w[1], w[2], w[3]));
                    oacc[db] = E::mfma(fr[i], b, oacc[db]);
                }
#pragma unroll
                for (int ch = chunk_lo(h, j); ch < chunk_lo(h, j + 1); ++ch) sm_chunk(h, ch);
                __builtin_amdgcn_sched_barrier(0);
            }
            sm_end(h);
        }
    };
    using std::integral_constant;
    constexpr integral_constant<int, 0> c0{};
    constexpr integral_constant<int, 1> c1{};
    constexpr integral_constant<int, 2> c2{};
    constexpr std::false_type no{};
    constexpr std::true_type yes{};

    if constexpr (kBN == 64) {
        // tile 0: both QK products, and the weights of its first block against that block's maximum
        {
            swap_barrier(0);
            next_addrs(0);
            if (!kLists && mask_tile == 0) {
                step(yes, c0, no, no, c0, no, no, c0, 0, 0, 0);
                mask_tail(0);
                step(no, c0, no, yes, c2, no, no, c0, 0, 0, 0);
            } else {
                step(yes, c0, no, yes, c2, no, no, c0, 0, 0, 0);
            }
        }
        // tile t >= 1, first half: QK(t, keys 0..31), weights of (t-1, keys 32..63), PV of (t-1, keys 0..31);
        // second half: QK(t, 32..63), weights of (t, 0..31), PV of (t-1, 32..63)
        auto tile_step = [&](auto check, auto kbuf, int t) {   // kbuf = t & 1, as a compile-time constant
            swap_barrier(t);
            next_addrs(t);
            step(yes, c1, yes, yes, c1, yes, check, kbuf, kbuf ^ 1, t - 1, t);
        };
        auto walk = [&](auto check) {
            int t = 1;   // (two steps per trip: the LDS buffers of every step are compile-time constants)
            for (; t + 1 < n_tiles; t += 2) {
                tile_step(check, c1, t);
                tile_step(check, c0, t + 1);
            }
            if (t < n_tiles) tile_step(check, c1, t);
            swap_barrier(n_tiles);
            step(no, c1, yes, no, c0, yes, check, c0, (n_tiles - 1) & 1, n_tiles - 1, n_tiles - 1);
        };
        if (!kLists && mask_tile >= 0) walk(yes);
        else walk(no);
    } else {
        // 32-key tiles: the step behind barrier b forms the scores of tile b, weights tile b-1 and adds
        // tile b-2 to O^T, all in the half (of S, pw and of the K and V buffers) of its parity.
        auto block_step = [&](auto check, auto par, auto qk, auto sm, auto pv, int b) {
            swap_barrier(b);
            next_addrs(b);
            if constexpr (decltype(par)::value == 0) step(qk, sm, pv, no, c0, no, check, c0, 0, b - 1, 0);
            else step(no, c0, no, qk, sm, pv, check, c1, 1, 0, b - 1);
        };
        auto walk = [&](auto check) {
            block_step(check, c0, yes, c0, no, 0);
            if (n_tiles > 1) block_step(check, c1, yes, c2, no, 1);
            else block_step(check, c1, no, c2, no, 1);
            int b = 2;
            for (; b + 1 < n_tiles; b += 2) {
                block_step(check, c0, yes, c1, yes, b);
                block_step(check, c1, yes, c1, yes, b + 1);
            }
            if (b < n_tiles) { block_step(check, c0, yes, c1, yes, b); ++b; }
            // here b = max(n_tiles, 2); the last tile still has to be weighted (unless it was the first) and added
            if (n_tiles >= 2) {
                if (b & 1) block_step(check, c1, no, c1, yes, b);
                else block_step(check, c0, no, c1, yes, b);
                ++b;
            }
            if (b & 1) block_step(check, c1, no, c0, yes, b);
            else block_step(check, c0, no, c0, yes, b);
        };
        if (!kLists && mask_tile >= 0) walk(yes);
        else walk(no);
    }

    // ---- epilogue: normalise, round to bf16, store ------------------------------------------
    // In the accumulator layout a lane holds 4 consecutive head dims (8 bytes) at a time of ITS
    // query; stored like that every store instruction would touch 64 different rows.  So each wave
    // turns its 32 x 128 output tile through 4 KiB of LDS, 64 head dims at a time: lanes write
    // their 8-byte pieces, then read back 16-byte chunks as (row = 8*i + lane/8, chunk = lane%8)
    // and store 8 rows x 128 contiguous bytes per instruction.  The K buffers are free by now (last
    // read before the final barrier, nothing in flight); a wave only touches its own 4 KiB, so
    // the only ordering needed is between its own LDS writes and reads.
    const float inv = 1.f / sum_across_halves(l_run);
    {
        uint8_t* stage = &sK[0][0] + wave * 4096;   // [32 rows][8 chunks of 16 B], chunk ^= row & 7
        const int srow = lane >> 3, schunk = lane & 7;
        uint64_t st_off[4];
        bool st_ok[4];
        const uint32_t o_pitch = (uint32_t)p.o_stride_n * 2u;   // O may have a token stride of its own
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = 8 * i + srow;
            st_ok[i] = !dense || q_first + row < p.n_dense_rows;
            if (MODE == kRagged) st_ok[i] = coord_inside(s_coord[q_first + row], q_limit);
            uint64_t off = q_row_off(row);
            if (o_pitch != row_pitch) {   // back to the row index (table entries are whole rows)
                const uint32_t r = dense ? (uint32_t)(off / row_pitch) : q_base + s_rowbytes[q_first + row] / row_pitch;
                off = (uint64_t)r * o_pitch;
            }
            st_off[i] = off + schunk * 16;
        }
        uint8_t* wr = stage + qcol * 128 + 8 * half;
#pragma unroll
        for (int pass = 0; pass < D / 64; ++pass) {
#pragma unroll
            for (int dbp = 0; dbp < 2; ++dbp)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    const f32x16& o = oacc[2 * pass + dbp];
                    uint2 v;
                    v.x = E::pack(o[4 * rq] * inv, o[4 * rq + 1] * inv);
                    v.y = E::pack(o[4 * rq + 2] * inv, o[4 * rq + 3] * inv);
                    *(uint2*)(wr + (((4 * dbp + rq) ^ (qcol & 7)) << 4)) = v;
                }
            __builtin_amdgcn_wave_barrier();   // (compiler: keep the reads below the writes above)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = 8 * i + srow;
                const uint4 x = *(const uint4*)(stage + row * 128 + ((schunk ^ (row & 7)) << 4));
                if (st_ok[i]) *(uint4*)((uint8_t*)Oh + st_off[i] + pass * 128) = x;
            }
            __builtin_amdgcn_wave_barrier();   // (... and the next pass's writes below these reads)
        }
    }
}

// The kernel: picks this workgroup's query tile and runs it.  Workgroups are dealt round-robin to the
// 8 XCDs; block b runs on XCD b % 8 as that XCD's (b / 8)-th workgroup.  The XCDs walk the heads
// TOGETHER: within a head every XCD owns one eighth of the head's tile order (a compact range of
// query groups; which eighth rotates from head to head, so that the short lists of border groups are
// spread evenly), so at any time the whole chip reads the K/V of one or two heads (which the memory-side
// cache holds) and every XCD's L2 sees a compact patch of neighbouring groups.  In joint mode the
// long-running dense tiles over the prompt rows get the lowest block indices, dealt round-robin over
// the XCDs, and the grouped tiles follow.
template <bool DENSE>
__device__ __forceinline__ bool head_sync_tile(const AttnParams& p, int xcd, int idx, int& bh, int& t_in_head) {
    const int per = DENSE ? p.per_xcd_dense : p.per_xcd;
    const int tph = DENSE ? p.q_tiles_dense : p.geo.num_groups * p.q_tiles;
    bh = (int)fdiv((uint32_t)idx, DENSE ? p.fd_per_xcd_dense : p.fd_per_xcd);
    t_in_head = ((xcd + bh) % kNumXcd) * per + (idx - bh * per);   // (rotated per head: border groups have shorter lists)
    return t_in_head < tph && bh < p.batch * p.heads;
}
// Small launches (p.longest_first; at most 64 groups): the hardware hands out workgroups in block order
// and a launch of only a few rounds of workgroups ends when its last long one does, so the groups with
// the longest lists go first and the short ones fill the tail.  Block b is query tile b % q_tiles of
// (batch, head) (b / q_tiles) % (batch * heads) of the group whose list is the (b / (q_tiles * batch *
// heads))-th longest (ties: lower id first); lane j ranks group j against the others, every wave for
// itself.
__device__ __forceinline__ bool longest_first_tile(const AttnParams& p, int b, int& bh, int& qt, int& gamma) {
    const int G = p.geo.num_groups;
    const int rank = (int)fdiv((uint32_t)b, p.fd_tiles_per_rank), rem = b - rank * p.batch * p.heads * p.q_tiles;
    if (rank >= G) return false;
    bh = (int)fdiv((uint32_t)rem, p.fd_q_tiles);
    qt = rem - bh * p.q_tiles;
    const int lane = threadIdx.x & 63;
    const int key = lane < G ? min(max(p.kv_count[lane], 0), p.max_kv) * 64 + (63 - lane) : -1;
    int r = 0;
#pragma unroll
    for (int k = 0; k < 64; ++k) r += __builtin_amdgcn_readlane(key, k) > key ? 1 : 0;
    const uint64_t m = __ballot(lane < G && r == rank);   // (the keys differ, so exactly one lane)
    gamma = __builtin_amdgcn_readfirstlane(__ffsll((long long)m) - 1);
    return true;
}

template <int NWAVES, int BN, int MODE, bool F16, int D>
__global__ __launch_bounds__(NWAVES * 64, 2) void attn_mfma_kernel(AttnParams p) {
    __shared__ __attribute__((aligned(1024))) uint8_t sK[2][BN * kRowBytes];
    __shared__ __attribute__((aligned(1024))) uint8_t sV[2][BN * kRowBytes];
    const int xcd = blockIdx.x % kNumXcd, idx = blockIdx.x / kNumXcd;
    int bh, t_in_head;
    if constexpr (MODE == kJoint) {
        const int dense_per_xcd = (p.n_dense_tiles + kNumXcd - 1) / kNumXcd;
        if (idx < dense_per_xcd) {
            const int tile = idx * kNumXcd + xcd;
            if (tile < p.n_dense_tiles) {
                bh = (int)fdiv((uint32_t)tile, p.fd_tiles_per_head_dense);
                attn_tile<NWAVES, BN, MODE, F16, D, true>(p, bh, tile - bh * p.q_tiles_dense, sK, sV);
            }
        } else if (p.longest_first) {
            int qt, gamma;
            if (longest_first_tile(p, (int)blockIdx.x - dense_per_xcd * kNumXcd, bh, qt, gamma))
                attn_tile<NWAVES, BN, MODE, F16, D, false>(p, bh, qt, sK, sV, gamma);
        } else if (head_sync_tile<false>(p, xcd, idx - dense_per_xcd, bh, t_in_head)) {
            attn_tile<NWAVES, BN, MODE, F16, D, false>(p, bh, t_in_head, sK, sV);
        }
    } else if (MODE != kDense && p.longest_first) {
        int qt, gamma;
        if (longest_first_tile(p, (int)blockIdx.x, bh, qt, gamma))
            attn_tile<NWAVES, BN, MODE, F16, D, false>(p, bh, qt, sK, sV, gamma);
    } else {
        if (head_sync_tile<MODE == kDense>(p, xcd, idx, bh, t_in_head))
            attn_tile<NWAVES, BN, MODE, F16, D, MODE == kDense>(p, bh, t_in_head, sK, sV);
    }
}

template <int NWAVES, int BN, bool F16, int D>
inline hipError_t launch_one(const AttnParams& p, int mode, hipStream_t stream) {
    const dim3 block(NWAVES * 64);
    const size_t dyn = mode == kDense ? 0 : sizeof(int32_t) * (mode == kRagged ? 2 : 1) * ((size_t)p.geo.group_tokens + p.max_kv);
    const int bh = p.batch * p.heads;
    const int grouped_blocks = kNumXcd * p.per_xcd * bh, dense_blocks = kNumXcd * p.per_xcd_dense * bh;
    if (mode == kRagged) {
        hipLaunchKernelGGL((attn_mfma_kernel<NWAVES, BN, kRagged, F16, D>), dim3(grouped_blocks), block, dyn, stream, p);
    } else if (mode == kDense) {
        if constexpr (NWAVES == 8)   // (the only tile height dense launches use)
            hipLaunchKernelGGL((attn_mfma_kernel<NWAVES, BN, kDense, F16, D>), dim3(dense_blocks), block, dyn, stream, p);
        else
            return hipErrorInvalidValue;
    } else if (mode == kGrouped) {
        hipLaunchKernelGGL((attn_mfma_kernel<NWAVES, BN, kGrouped, F16, D>), dim3(grouped_blocks), block, dyn, stream, p);
    } else {
        if constexpr (BN == 64) {
            const int blocks = xcd_padded_blocks(p.n_dense_tiles) + grouped_blocks;
            hipLaunchKernelGGL((attn_mfma_kernel<NWAVES, BN, kJoint, F16, D>), dim3(blocks), block, dyn, stream, p);
        } else {
            return hipErrorInvalidValue;
        }
    }
    return hipGetLastError();
}

// p.q_tiles (and p.q_tiles_dense) were computed by the host for the query-tile height chosen here:
// 256, 128 or 64 rows.  64-row workgroups take 32-key tiles unless the lists are long.
template <bool F16, int D>
inline hipError_t launch_by_tile(const AttnParams& p, int mode, hipStream_t stream) {
    const int bm = mode == kDense ? 256 : (p.geo.group_tokens / p.q_tiles);
    if (bm == 256) return launch_one<8, 64, F16, D>(p, mode, stream);
    if (bm == 128) return launch_one<4, 64, F16, D>(p, mode, stream);
    // (measured at 512x512 tokens in 8x8 groups: lists of 9 / 25 / 49 groups gain 16-19 % from the small
    // tiles, the criss-cross lists of 127 groups lose 5 %)
    // (not for joint sequences: that variant of the 32-key schedule does not fit the register file)
    if (mode != kJoint && (int64_t)p.max_kv * p.geo.group_tokens <= 64 * 64) return launch_one<2, 32, F16, D>(p, mode, stream);
    return launch_one<2, 64, F16, D>(p, mode, stream);
}

}  // namespace grat
