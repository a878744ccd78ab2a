// Internal declarations shared by the host entry points and the kernels of libgrat.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fastdiv.h"
#include "grat.h"

namespace grat {

// Grid / group geometry normalised to three axes (missing leading axes have extent 1).
struct Geometry {
    int32_t T[3];   // token grid
    int32_t g[3];   // tokens per group along each axis
    int32_t G[3];   // groups along each axis, ceil(T/g)
    int32_t num_groups;
    int32_t group_tokens;  // g0*g1*g2
    int64_t n_tokens;
};

struct AttnParams {
    const void* Q;
    const void* K;
    const void* V;
    void* O;
    int64_t stride_b, stride_h;      // Q, K, V: elements between batches / heads
    int32_t stride_n;                // ... between tokens
    int64_t o_stride_b, o_stride_h;  // the same for O
    int32_t o_stride_n;
    int32_t batch, heads;
    float scale_log2;          // scale * log2(e)
    Geometry geo;
    const int32_t* kv_count;
    const int32_t* kv_index;
    int32_t max_kv;
    int32_t n_tokens;          // dense tiles: number of KV rows (the whole sequence)
    int32_t q_tiles;           // query tiles per group
    int32_t total_tiles;       // batch * heads * groups * q_tiles (grouped) or batch * heads * q_tiles_dense (dense)
    int32_t strip_w;           // grouped bf16 path: query groups are walked in column strips this wide
    // dense tiles (dense entry point, and the prompt rows of a joint sequence)
    int32_t q_tiles_dense;     // query tiles per head
    int32_t n_dense_rows;      // query rows per head
    int32_t dense_row0;        // first of them
    int32_t n_dense_tiles;     // joint sequence: batch * heads * q_tiles_dense, launched ahead of the grouped tiles
    // joint sequence (prompt tokens + grid tokens)
    int32_t n_global;          // prompt tokens
    int32_t global_row0;       // first prompt row
    int32_t grid_row0;         // first grid row
    // MFMA kernel: host-prepared divisors for the index decompositions of its prologue
    FastDiv fd_tiles_per_head_dense;  // by q_tiles_dense
    FastDiv fd_heads, fd_q_tiles;
    int32_t per_xcd, per_xcd_dense;   // tiles of one head that one XCD owns: ceil(tiles per head / 8), grouped and dense
    FastDiv fd_per_xcd, fd_per_xcd_dense;
    int32_t longest_first;            // small grouped launches: tiles are handed out by list length, longest first
    FastDiv fd_tiles_per_rank;        // by batch * heads * q_tiles
    FastDiv fd_strip, fd_strip_w, fd_strip_tail;   // strip order: by rows * strip_w, strip_w, width of the last strip
    int32_t strip_full;               // full strips: cols / strip_w
    FastDiv fd_g1, fd_g2, fd_G1, fd_G2;            // token in group -> box coordinates, group id -> group coordinates
};

// What a workgroup of the MFMA attention kernel can be (its MODE template argument).
//   kGrouped  every workgroup is a query tile of one group and walks that group's KV list;
//   kDense    every workgroup is a tile of consecutive query rows and walks all KV tiles;
//   kJoint    joint sequence of prompt tokens and grid tokens: the first p.n_dense_tiles tiles are
//             dense tiles over the prompt rows (they attend the whole sequence), the others are
//             grouped tiles whose walk starts with the prompt tokens' KV tiles.
//   kRagged   kGrouped for a grid the group dims do not divide (Eq. 2-4 are floor divisions): a
//             group at the far border is the part of its box inside the grid.  Boxes are still
//             walked whole; tokens of a box that fall outside the grid are fetched from a clamped
//             (valid, meaningless) address and get weight 0, queries outside are not stored.
enum AttnMode : int { kGrouped = 0, kDense = 1, kJoint = 2, kRagged = 3 };

// Launchers: each returns the hipError_t of its launch.
hipError_t launch_build_block_lists(const Geometry& geo, int ndim, grat_pattern pattern,
                                    const int32_t radius[3], int32_t* d_kv_count,
                                    int32_t* d_kv_index, int32_t max_kv, hipStream_t stream);
hipError_t launch_validate_block_lists(const Geometry& geo, const int32_t* d_kv_count, const int32_t* d_kv_index,
                                       int32_t max_kv, int32_t* d_status, hipStream_t stream);
hipError_t launch_attn_f32(const AttnParams& p, int head_dim, bool dense, hipStream_t stream);
hipError_t launch_attn_bf16(const AttnParams& p, int mode /* AttnMode */, bool f16, int head_dim, hipStream_t stream);

// Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).
constexpr int kNumXcd = 8;
// fp32 kernel: every XCD gets one contiguous range of the logical tile order.
__device__ __forceinline__ int xcd_contiguous_tile(int block, int total) {
    const int per = (total + kNumXcd - 1) / kNumXcd;
    return (block % kNumXcd) * per + block / kNumXcd;   // may be >= total: caller exits
}
inline int xcd_padded_blocks(int total) { return ((total + kNumXcd - 1) / kNumXcd) * kNumXcd; }

// Order in which the query groups of one head are handed to consecutive workgroups: column strips
// of the group grid, `strip_w` groups wide, each walked row by row.  The ~32 workgroups an XCD
// runs at a time then cover a compact 2D patch of groups (4 rows x 8 columns for strip_w = 8)
// whose K/V neighbourhoods overlap in both directions, instead of one long group-row.
// rows = all leading group axes flattened, cols = the last group axis; returns the linear group id.
__device__ __forceinline__ int strip_order_group_fast(uint32_t u, int rows, int cols, const AttnParams& p) {
    uint32_t s = fdiv(u, p.fd_strip);
    int w = p.strip_w;
    FastDiv fw = p.fd_strip_w;
    if ((int)s >= p.strip_full) { s = p.strip_full; w = cols - p.strip_full * p.strip_w; fw = p.fd_strip_tail; }
    const uint32_t v = u - s * (uint32_t)(rows * p.strip_w);
    const uint32_t vq = fdiv(v, fw);
    return (int)(vq * cols + s * p.strip_w + (v - vq * w));
}
__device__ __forceinline__ int strip_order_group(int u, int rows, int cols, int strip_w) {
    const int full = cols / strip_w;
    int s = u / (rows * strip_w), w = strip_w;
    if (s >= full) { s = full; w = cols - full * strip_w; }
    const int v = u - s * rows * strip_w;
    return (v / w) * cols + s * strip_w + v % w;
}

}  // namespace grat
