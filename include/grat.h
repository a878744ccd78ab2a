/*
 * libgrat — GRAT grouped sparse attention (forward) for AMD MI355X (gfx950), C ABI.
 *
 * The method (GRAT, arXiv 2505.14687, Sec. 3.2): image or video tokens laid out
 * row-major over a 2D / 3D grid are partitioned into non-overlapping groups (Eq. 2-4, 9-11);
 * every query of a group attends the same set of key/value groups — the surrounding blocks
 * (GRAT-B, Eq. 5-6 / 12-13) or the criss-cross region (GRAT-X, Eq. 7-8 / 14-15) — and the
 * output is exactly softmax attention (Sec. 3.1, Eq. 1) restricted to that set.
 *
 * Conventions shared by every entry point
 *   - Plain C: pointers and sizes only.  Pointers named d_* and the Q/K/V/O tensors are DEVICE
 *     pointers (memory of the current HIP device); `grid`, `group`, `radius` and the out
 *     parameters of grat_block_list_shape are HOST pointers, read before the call returns.
 *   - The caller owns every buffer.  The library allocates nothing, frees nothing, never
 *     synchronises the device: work is enqueued on `hip_stream` (a hipStream_t, NULL = the
 *     default stream) and the call returns.
 *   - Errors are return codes.  All argument checks run on the host before anything is
 *     launched, so a non-zero status other than GRAT_ERR_HIP means no work was enqueued.
 *   - Token layout: token (x0, .., x_{ndim-1}) of the grid is row ((x0*T1)+x1)*T2+x2 of the
 *     sequence (last dim fastest).  Grouping is index arithmetic inside the kernels; no
 *     permuted copy of Q/K/V is ever made.
 *   - Group ids: group (p0, .., p_{ndim-1}) has linear id ((p0*G1)+p1)*G2+p2 with
 *     G_k = ceil(T_k / g_k).
 *   - Tensors are addressed as  base + b*stride_b + h*stride_h + n*stride_n + c  (strides in
 *     ELEMENTS, the head_dim axis contiguous), so [B][H][N][d] and [B][N][H][d] both work.
 *     Q, K, V and O share one set of strides.
 */
#ifndef GRAT_H
#define GRAT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GRAT_OK = 0,
    GRAT_ERR_NULL = 1,             /* a required pointer is NULL                               */
    GRAT_ERR_BAD_DIMS = 2,         /* ndim not in 1..3, a non-positive extent, negative radius,
                                      non-positive scale, strides that make rows overlap        */
    GRAT_ERR_INDIVISIBLE = 3,      /* joint sequences only: a group dim does not divide its grid dim */
    GRAT_ERR_BAD_PATTERN = 4,
    GRAT_ERR_BUFFER_TOO_SMALL = 5, /* max_kv smaller than the longest list                      */
    GRAT_ERR_UNSUPPORTED = 6,      /* shape / dtype outside what the kernels cover (see below)  */
    GRAT_ERR_HIP = 7               /* a HIP runtime call or the launch itself failed            */
} grat_status;

typedef enum {
    /* Eq. 5-6 / 12-13: KV group p' is attendable iff |p'_k - p_k| <= radius[k] on every axis;
       neighbours outside the grid are dropped (no wrap-around, no window shift). */
    GRAT_BLOCK = 0,
    /* GRAT-X as the prose of Sec. 3.2 states it: the KV groups on the axis lines through the
       query group, i.e. at least ndim-1 group coordinates equal.  2D: its group-row and
       group-column (Eq. 7-8 with the printed "n = p" read as "n = q"). */
    GRAT_CROSS = 1,
    /* Eq. 14-15 as printed: at least ONE group coordinate equal (three planes in 3D).
       Identical to GRAT_CROSS for ndim == 2. */
    GRAT_CROSS_PLANES = 2,
    /* every group attends every group (Eq. 1) */
    GRAT_DENSE = 3
} grat_pattern;

/* element type of Q, K, V and O: bfloat16, IEEE binary32, IEEE binary16 */
typedef enum { GRAT_BF16 = 0, GRAT_F32 = 1, GRAT_F16 = 2 } grat_dtype;

/*
 * Sizes of the block lists for a pattern (host only, touches no GPU).
 *   ndim              1, 2 or 3
 *   grid[ndim]        token grid T_k            (host)
 *   group[ndim]       tokens per group g_k      (host); a ragged last group is allowed here
 *   radius[ndim]      per-axis b_k for GRAT_BLOCK (host); ignored (may be NULL) otherwise
 *   num_groups (out)  G = prod G_k
 *   max_kv     (out)  length of the longest list:  prod min(2 b_k + 1, G_k)  for BLOCK,
 *                     sum G_k - (ndim - 1) for CROSS,  G - prod (G_k - 1) for CROSS_PLANES,
 *                     G for DENSE
 */
grat_status grat_block_list_shape(int32_t ndim, const int32_t* grid, const int32_t* group,
                                  grat_pattern pattern, const int32_t* radius,
                                  int32_t* num_groups, int32_t* max_kv);

/*
 * Build the per-query-group lists of attendable KV groups on the GPU (Sec. 3.2, Eq. 5-8 and
 * Eq. 12-15; the role the block mask plays in the paper's own implementation).
 *   d_kv_count[G]          (device, out) list length of every query group, >= 1
 *   d_kv_index[G * max_kv] (device, out) row gamma holds that group's KV group ids in
 *                          ascending order, then -1 padding up to max_kv
 *   max_kv                 row pitch of d_kv_index; GRAT_ERR_BUFFER_TOO_SMALL if it is less
 *                          than what grat_block_list_shape reports
 * Other arguments as in grat_block_list_shape.  Asynchronous on hip_stream.
 */
grat_status grat_build_block_lists(int32_t ndim, const int32_t* grid, const int32_t* group,
                                   grat_pattern pattern, const int32_t* radius,
                                   int32_t* d_kv_count, int32_t* d_kv_index, int32_t max_kv,
                                   void* hip_stream);

/*
 * Check block lists against the format grat_build_block_lists writes, on the GPU: for callers that
 * make their own lists (any set of KV groups per query group is a valid instance of the attendable
 * sets of Sec. 3.2, Eq. 5-8 / 12-15, as long as it has this format).  The attention entry points do
 * not check lists themselves; they only force counts and entries into range.
 *   d_kv_count[G], d_kv_index[G * max_kv]  (device, in) the lists, G = prod ceil(grid[k] / group[k])
 *   d_status[1]  (device, out) 0 if every list is well formed, else the OR of
 *                GRAT_LIST_BAD_COUNT    a count outside [1, max_kv]
 *                GRAT_LIST_BAD_ENTRY    a used entry outside [0, G)
 *                GRAT_LIST_BAD_PADDING  an entry behind a list's count that is not -1
 *                (order of the entries is not checked: any order gives the same attention result)
 * Errors: GRAT_ERR_NULL, the geometry errors of grat_block_list_shape, GRAT_ERR_BUFFER_TOO_SMALL
 * (max_kv < 1), GRAT_ERR_HIP.  Asynchronous on hip_stream (two small launches, no memset, nothing
 * allocated): read d_status after synchronising with the stream.
 */
enum { GRAT_LIST_BAD_COUNT = 1, GRAT_LIST_BAD_ENTRY = 2, GRAT_LIST_BAD_PADDING = 4 };
grat_status grat_validate_block_lists(int32_t ndim, const int32_t* grid, const int32_t* group,
                                      const int32_t* d_kv_count, const int32_t* d_kv_index,
                                      int32_t max_kv, int32_t* d_status, void* hip_stream);

/*
 * O = softmax(scale * Q K^T restricted to the block lists) V, per batch and head
 * (Sec. 3.1 Eq. 1 over the attendable sets of Sec. 3.2).
 *   Q, K, V (device, in), O (device, out): `dtype` elements, addressed with the strides
 *                          above; O must not alias Q, K or V
 *   batch, heads, head_dim tensor extents; the sequence length is prod grid[k]
 *   scale                  > 0, multiplies Q K^T (the paper uses 1/sqrt(head_dim))
 *   ndim, grid, group      as above.  group[k] need not divide grid[k]: Eq. 2-4 / 9-11 are floor
 *                          divisions, so the groups at the far border are the part of their
 *                          box that lies inside the grid (lists as grat_build_block_lists
 *                          writes them for the same grid and group)
 *   d_kv_count, d_kv_index, max_kv   lists in the format grat_build_block_lists writes (the
 *                          caller may also supply its own).  Every used entry must lie in
 *                          [0, G) and every count in [1, max_kv]: the result for a list that
 *                          breaks this is undefined (the kernels force counts and entries into
 *                          range so that no access leaves the tensors, nothing more);
 *                          grat_validate_block_lists checks a list on the GPU.
 * Supported (GRAT_ERR_UNSUPPORTED otherwise):
 *   GRAT_BF16, GRAT_F16: head_dim 128 or 64, tokens per (whole) group a multiple of 64; with clipped border
 *              groups also group[k] <= 1024 on the last two axes;
 *   GRAT_F32 : head_dim 64 or 128, any group size;
 *   all      : N < 2^31 tokens, stride_n < 2^24 elements, max_kv <= 8192; 16-bit types also: the
 *              rows of one group span less than 4 GiB (first to last token of a group, in bytes).
 *              The tensors themselves may exceed 4 GiB: a packed [B][N][3][H][d] buffer of a long
 *              sequence is passed as three pointers into it with stride_n = 3 * H * d.
 * 16-bit paths: scores, running max / sum and the output accumulator are fp32; softmax weights
 * are rounded to the element type (nearest-even) before multiplying V; O is rounded once.
 * Asynchronous on hip_stream.
 */
grat_status grat_attention_fwd(const void* Q, const void* K, const void* V, void* O,
                               grat_dtype dtype, int32_t batch, int32_t heads, int32_t head_dim,
                               int64_t stride_b, int64_t stride_h, int64_t stride_n, float scale,
                               int32_t ndim, const int32_t* grid, const int32_t* group,
                               const int32_t* d_kv_count, const int32_t* d_kv_index,
                               int32_t max_kv, void* hip_stream);

/*
 * The same for a JOINT sequence of prompt tokens and grid tokens, as the diffusion transformers the
 * method is applied to use (the method section, Sec. 3.2, defines the spatial part only; the
 * sparsities printed in its ablation table count 512 always-attended prompt tokens).
 *   n_global      >= 0 prompt ("global") tokens; the sequence has n_global + prod grid[k] rows
 *   global_first  non-zero: the prompt tokens are rows [0, n_global) and the grid tokens follow;
 *                 zero: the grid tokens come first
 * A grid query attends the KV groups of its list plus every prompt token; a prompt query attends
 * the whole sequence.  Everything else as in grat_attention_fwd (which is the n_global = 0 case).
 * Supported: GRAT_BF16 and GRAT_F16 (GRAT_F32 only with n_global = 0); with n_global > 0 every group[k] must
 * divide grid[k] (GRAT_ERR_INDIVISIBLE otherwise).
 */
grat_status grat_attention_global_fwd(const void* Q, const void* K, const void* V, void* O,
                                      grat_dtype dtype, int32_t batch, int32_t heads,
                                      int32_t head_dim, int64_t stride_b, int64_t stride_h,
                                      int64_t stride_n, float scale, int32_t n_global,
                                      int32_t global_first, int32_t ndim, const int32_t* grid,
                                      const int32_t* group, const int32_t* d_kv_count,
                                      const int32_t* d_kv_index, int32_t max_kv, void* hip_stream);

/*
 * The same again for Q, K and V that were never split: QKV is the output of a fused projection,
 * one buffer [batch][n_global + N][3][heads][head_dim] (Q, K, V of a token side by side), and O is
 * [batch][n_global + N][heads][head_dim], both contiguous.  Nothing is copied: the kernels read the
 * three tensors through the token stride 3 * heads * head_dim.  n_global = 0 for a plain grid
 * sequence.  Everything else, limits included, as in grat_attention_global_fwd.
 */
grat_status grat_attention_packed_fwd(const void* QKV, void* O, grat_dtype dtype, int32_t batch,
                                      int32_t heads, int32_t head_dim, float scale, int32_t n_global,
                                      int32_t global_first, int32_t ndim, const int32_t* grid,
                                      const int32_t* group, const int32_t* d_kv_count,
                                      const int32_t* d_kv_index, int32_t max_kv, void* hip_stream);

/*
 * Full attention (Sec. 3.1, Eq. 1) over n_tokens tokens with the same tiling and arithmetic as
 * grat_attention_fwd: the comparison point for speedups.  Any n_tokens >= 1.
 * Supported dtypes / head_dim as above.
 */
grat_status grat_dense_attention_fwd(const void* Q, const void* K, const void* V, void* O,
                                     grat_dtype dtype, int32_t batch, int32_t heads,
                                     int64_t n_tokens, int32_t head_dim, int64_t stride_b,
                                     int64_t stride_h, int64_t stride_n, float scale,
                                     void* hip_stream);

/* Static, NUL-terminated description of a status code. */
const char* grat_status_string(grat_status status);

#ifdef __cplusplus
}
#endif
#endif /* GRAT_H */
