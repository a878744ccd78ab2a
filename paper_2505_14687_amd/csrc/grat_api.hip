// Host side of libgrat: argument validation and dispatch.  No allocation, no synchronisation.
#include <cmath>
#include <cstdint>

#include "grat_common.h"

namespace grat {
namespace {

constexpr int64_t kMaxElems = (int64_t)1 << 31;
constexpr int32_t kMaxListLen = 8192;

// Validate (ndim, grid, group) and normalise to three axes by prepending unit axes.
grat_status make_geometry(int32_t ndim, const int32_t* grid, const int32_t* group, Geometry* out) {
    if (!grid || !group) return GRAT_ERR_NULL;
    if (ndim < 1 || ndim > 3) return GRAT_ERR_BAD_DIMS;
    Geometry geo;
    int64_t n = 1, ng = 1, G = 1;
    for (int k = 0; k < 3; ++k) {
        const int src = k - (3 - ndim);
        const int32_t T = src >= 0 ? grid[src] : 1;
        const int32_t g = src >= 0 ? group[src] : 1;
        if (T < 1 || g < 1) return GRAT_ERR_BAD_DIMS;
        geo.T[k] = T;
        geo.g[k] = g;
        geo.G[k] = (T + g - 1) / g;
        n *= T;
        ng *= g;
        G *= geo.G[k];
        if (n >= kMaxElems || ng >= kMaxElems) return GRAT_ERR_BAD_DIMS;
    }
    geo.n_tokens = n;
    geo.group_tokens = (int32_t)ng;
    geo.num_groups = (int32_t)G;
    *out = geo;
    return GRAT_OK;
}

grat_status make_radius(int32_t ndim, grat_pattern pattern, const int32_t* radius, int32_t out[3]) {
    out[0] = out[1] = out[2] = 0;
    if (pattern != GRAT_BLOCK) return GRAT_OK;
    if (!radius) return GRAT_ERR_NULL;
    for (int k = 0; k < ndim; ++k) {
        if (radius[k] < 0) return GRAT_ERR_BAD_DIMS;
        out[k + (3 - ndim)] = radius[k];
    }
    return GRAT_OK;
}

bool valid_pattern(grat_pattern p) {
    return p == GRAT_BLOCK || p == GRAT_CROSS || p == GRAT_CROSS_PLANES || p == GRAT_DENSE;
}

int64_t longest_list(const Geometry& geo, int32_t ndim, grat_pattern pattern, const int32_t r[3]) {
    const int first = 3 - ndim;
    int64_t v;
    switch (pattern) {
        case GRAT_BLOCK:
            v = 1;
            for (int k = first; k < 3; ++k) v *= std::min<int64_t>(2 * (int64_t)r[k] + 1, geo.G[k]);
            return v;
        case GRAT_CROSS:
            v = -(ndim - 1);
            for (int k = first; k < 3; ++k) v += geo.G[k];
            return v;
        case GRAT_CROSS_PLANES:
            v = 1;
            for (int k = first; k < 3; ++k) v *= geo.G[k] - 1;
            return geo.num_groups - v;
        default:
            return geo.num_groups;
    }
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }
bool is16(grat_dtype t) { return t == GRAT_BF16 || t == GRAT_F16; }   // the MFMA path's element types

// O's strides when they are not Q's: same rules as in check_tensors.
grat_status check_out_strides(grat_dtype dtype, int32_t head_dim, int64_t b, int64_t h, int64_t n) {
    if (n < head_dim || b < 0 || h < 0) return GRAT_ERR_BAD_DIMS;
    const int vec = is16(dtype) ? 8 : 4;
    if (n % vec || b % vec || h % vec) return GRAT_ERR_UNSUPPORTED;
    if (n >= ((int64_t)1 << 24) || b >= ((int64_t)1 << 46) || h >= ((int64_t)1 << 46)) return GRAT_ERR_UNSUPPORTED;
    return GRAT_OK;
}

// Checks shared by the grouped and the dense attention entry points.
grat_status check_tensors(const void* Q, const void* K, const void* V, void* O, grat_dtype dtype,
                          int32_t batch, int32_t heads, int32_t head_dim, int64_t n_tokens,
                          int64_t stride_b, int64_t stride_h, int64_t stride_n, float scale) {
    if (!Q || !K || !V || !O) return GRAT_ERR_NULL;
    if (batch < 1 || heads < 1 || head_dim < 1 || n_tokens < 1) return GRAT_ERR_BAD_DIMS;
    if (!(scale > 0.f) || !std::isfinite(scale)) return GRAT_ERR_BAD_DIMS;
    if (stride_n < head_dim || stride_b < 0 || stride_h < 0) return GRAT_ERR_BAD_DIMS;
    if (!is16(dtype) && dtype != GRAT_F32) return GRAT_ERR_UNSUPPORTED;
    if (is16(dtype) && head_dim != 64 && head_dim != 128) return GRAT_ERR_UNSUPPORTED;
    if (dtype == GRAT_F32 && head_dim != 64 && head_dim != 128) return GRAT_ERR_UNSUPPORTED;
    // rows are read and written as 16-byte vectors
    const int vec = is16(dtype) ? 8 : 4;
    if (stride_n % vec || stride_b % vec || stride_h % vec) return GRAT_ERR_UNSUPPORTED;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O)) return GRAT_ERR_UNSUPPORTED;
    // the token stride is kept in 32 bits (a 64-row tile then spans less than 4 GiB); the tensor
    // itself may be larger than that: row addresses are formed in 64 bits
    if (stride_n >= ((int64_t)1 << 24)) return GRAT_ERR_UNSUPPORTED;
    if (stride_b >= ((int64_t)1 << 46) || stride_h >= ((int64_t)1 << 46)) return GRAT_ERR_UNSUPPORTED;
    if ((int64_t)batch * heads >= ((int64_t)1 << 24)) return GRAT_ERR_UNSUPPORTED;
    return GRAT_OK;
}

}  // namespace
}  // namespace grat

using namespace grat;

extern "C" grat_status grat_block_list_shape(int32_t ndim, const int32_t* grid, const int32_t* group,
                                             grat_pattern pattern, const int32_t* radius,
                                             int32_t* num_groups, int32_t* max_kv) {
    if (!num_groups || !max_kv) return GRAT_ERR_NULL;
    Geometry geo;
    grat_status st = make_geometry(ndim, grid, group, &geo);
    if (st != GRAT_OK) return st;
    if (!valid_pattern(pattern)) return GRAT_ERR_BAD_PATTERN;
    int32_t r[3];
    st = make_radius(ndim, pattern, radius, r);
    if (st != GRAT_OK) return st;
    *num_groups = geo.num_groups;
    *max_kv = (int32_t)longest_list(geo, ndim, pattern, r);
    return GRAT_OK;
}

extern "C" grat_status grat_build_block_lists(int32_t ndim, const int32_t* grid, const int32_t* group,
                                              grat_pattern pattern, const int32_t* radius,
                                              int32_t* d_kv_count, int32_t* d_kv_index,
                                              int32_t max_kv, void* hip_stream) {
    if (!d_kv_count || !d_kv_index) return GRAT_ERR_NULL;
    Geometry geo;
    grat_status st = make_geometry(ndim, grid, group, &geo);
    if (st != GRAT_OK) return st;
    if (!valid_pattern(pattern)) return GRAT_ERR_BAD_PATTERN;
    int32_t r[3];
    st = make_radius(ndim, pattern, radius, r);
    if (st != GRAT_OK) return st;
    if (max_kv < longest_list(geo, ndim, pattern, r)) return GRAT_ERR_BUFFER_TOO_SMALL;
    if ((int64_t)geo.num_groups * max_kv >= kMaxElems) return GRAT_ERR_UNSUPPORTED;
    const hipError_t e = launch_build_block_lists(geo, ndim, pattern, r, d_kv_count, d_kv_index,
                                                  max_kv, (hipStream_t)hip_stream);
    return e == hipSuccess ? GRAT_OK : GRAT_ERR_HIP;
}

extern "C" grat_status grat_validate_block_lists(int32_t ndim, const int32_t* grid, const int32_t* group,
                                                 const int32_t* d_kv_count, const int32_t* d_kv_index,
                                                 int32_t max_kv, int32_t* d_status, void* hip_stream) {
    if (!d_kv_count || !d_kv_index || !d_status) return GRAT_ERR_NULL;
    Geometry geo;
    const grat_status st = make_geometry(ndim, grid, group, &geo);
    if (st != GRAT_OK) return st;
    if (max_kv < 1) return GRAT_ERR_BUFFER_TOO_SMALL;
    if ((int64_t)geo.num_groups * max_kv >= kMaxElems) return GRAT_ERR_UNSUPPORTED;
    const hipError_t e = launch_validate_block_lists(geo, d_kv_count, d_kv_index, max_kv, d_status,
                                                     (hipStream_t)hip_stream);
    return e == hipSuccess ? GRAT_OK : GRAT_ERR_HIP;
}

// Divisors of the MFMA kernel's index decompositions, from the finished launch parameters.
static void fill_fastdivs(AttnParams& p) {
    const Geometry& geo = p.geo;
    p.per_xcd = (geo.num_groups * p.q_tiles + kNumXcd - 1) / kNumXcd;
    p.per_xcd_dense = (p.q_tiles_dense + kNumXcd - 1) / kNumXcd;
    p.fd_per_xcd = make_fastdiv((uint32_t)p.per_xcd);
    p.fd_per_xcd_dense = make_fastdiv((uint32_t)p.per_xcd_dense);
    p.fd_tiles_per_head_dense = make_fastdiv((uint32_t)p.q_tiles_dense);
    p.fd_heads = make_fastdiv((uint32_t)p.heads);
    p.fd_q_tiles = make_fastdiv((uint32_t)p.q_tiles);
    const int rows = geo.G[0] * geo.G[1], cols = geo.G[2], sw = p.strip_w > 0 ? p.strip_w : 1;
    p.strip_full = cols / sw;
    p.fd_strip = make_fastdiv((uint32_t)rows * (uint32_t)sw);
    p.fd_strip_w = make_fastdiv((uint32_t)sw);
    p.fd_strip_tail = make_fastdiv((uint32_t)(cols - p.strip_full * sw));   // (0 becomes 1: no tail strip, never used)
    p.fd_g1 = make_fastdiv((uint32_t)geo.g[1]);
    p.fd_g2 = make_fastdiv((uint32_t)geo.g[2]);
    p.fd_G1 = make_fastdiv((uint32_t)geo.G[1]);
    p.fd_G2 = make_fastdiv((uint32_t)geo.G[2]);
}

struct OutStrides { int64_t b, h, n; };   // O's own strides (elements)

// LDS the MFMA kernel needs beside its four 16-KiB tiles: the row-offset table of a group and the
// list's group origins, twice that with clipped border groups (box coordinates, in-grid limits).
static bool tables_fit_lds(const Geometry& geo, int32_t max_kv, bool ragged) {
    const int64_t tables = (ragged ? 2 : 1) * ((int64_t)geo.group_tokens + max_kv) * (int64_t)sizeof(int32_t);
    return 4 * 16384 + tables <= 160 * 1024;
}

// Shared by grat_attention_fwd (n_global = 0), grat_attention_global_fwd and grat_attention_packed_fwd.
static grat_status attention_fwd(const void* Q, const void* K, const void* V, void* O,
                                 grat_dtype dtype, int32_t batch, int32_t heads, int32_t head_dim,
                                 int64_t stride_b, int64_t stride_h, int64_t stride_n,
                                 OutStrides os, float scale,
                                 int32_t n_global, int32_t global_first, int32_t ndim,
                                 const int32_t* grid, const int32_t* group,
                                 const int32_t* d_kv_count, const int32_t* d_kv_index,
                                 int32_t max_kv, void* hip_stream) {
    if (!d_kv_count || !d_kv_index) return GRAT_ERR_NULL;
    Geometry geo;
    grat_status st = make_geometry(ndim, grid, group, &geo);
    if (st != GRAT_OK) return st;
    if (n_global < 0) return GRAT_ERR_BAD_DIMS;
    const int64_t seq_len = geo.n_tokens + n_global;
    if (seq_len >= kMaxElems) return GRAT_ERR_BAD_DIMS;
    st = check_tensors(Q, K, V, O, dtype, batch, heads, head_dim, seq_len, stride_b, stride_h,
                       stride_n, scale);
    if (st != GRAT_OK) return st;
    st = check_out_strides(dtype, head_dim, os.b, os.h, os.n);
    if (st != GRAT_OK) return st;
    bool ragged = false;   // a group dim does not divide its grid dim: groups at the far border are clipped
    for (int k = 0; k < 3; ++k) ragged = ragged || geo.T[k] % geo.g[k] != 0;
    if (ragged && n_global > 0) return GRAT_ERR_INDIVISIBLE;   // joint sequences: whole groups only
    if (max_kv < 1) return GRAT_ERR_BUFFER_TOO_SMALL;
    if (max_kv > kMaxListLen) return GRAT_ERR_UNSUPPORTED;
    if (n_global > 0 && !is16(dtype)) return GRAT_ERR_UNSUPPORTED;

    AttnParams p{};
    p.Q = Q; p.K = K; p.V = V; p.O = O;
    p.stride_b = stride_b; p.stride_h = stride_h; p.stride_n = (int32_t)stride_n;
    p.o_stride_b = os.b; p.o_stride_h = os.h; p.o_stride_n = (int32_t)os.n;
    p.batch = batch; p.heads = heads;
    p.scale_log2 = scale * 1.4426950408889634f;
    p.geo = geo;
    p.kv_count = d_kv_count; p.kv_index = d_kv_index; p.max_kv = max_kv;
    p.n_tokens = (int32_t)seq_len;

    const int n_g = geo.group_tokens;
    int bm;   // query rows per workgroup
    if (is16(dtype)) {
        if (n_g % 64) return GRAT_ERR_UNSUPPORTED;
        // byte offsets inside one group are kept in 32 bits
        const int64_t span_rows = (int64_t)(geo.g[0] - 1) * geo.T[1] * geo.T[2] + (int64_t)(geo.g[1] - 1) * geo.T[2] + geo.g[2];
        if (span_rows * stride_n * 2 >= ((int64_t)1 << 32)) return GRAT_ERR_UNSUPPORTED;
        if (n_g > 4096) return GRAT_ERR_UNSUPPORTED;   // intra-group offset table lives in LDS
        if (!tables_fit_lds(geo, max_kv, ragged)) return GRAT_ERR_UNSUPPORTED;
        bm = n_g % 256 == 0 ? 256 : (n_g % 128 == 0 ? 128 : 64);
        // A launch of fewer than two rounds of 256-row workgroups (one per compute unit) runs as 128-row
        // workgroups, two per compute unit, so that one's prologue and epilogue lie under the other's
        // walk (measured: +5 % at 64x64 tokens, nothing either way from 128x128 tokens on).
        if (bm == 256 && (int64_t)batch * heads * geo.num_groups < 2 * 256) bm = 128;
    } else {
        bm = 64;
    }
    p.q_tiles = (n_g + bm - 1) / bm;
    p.strip_w = geo.G[2] >= 16 ? 8 : geo.G[2];
    // (the launch pads every head's tiles to a multiple of 8: up to 7 more per head)
    const int64_t total = (int64_t)batch * heads * geo.num_groups * p.q_tiles;
    if ((int64_t)batch * heads * ((int64_t)geo.num_groups * p.q_tiles + 8) >= kMaxElems - 8) return GRAT_ERR_UNSUPPORTED;
    p.total_tiles = (int32_t)total;

    int mode = ragged ? kRagged : kGrouped;
    // the clipped-box tests of the bf16 kernel pack box coordinates into 12 + 10 + 10 bits
    if (ragged && is16(dtype) && (geo.g[1] > 1024 || geo.g[2] > 1024)) return GRAT_ERR_UNSUPPORTED;
    if (n_global > 0) {   // joint sequence: prompt rows become dense tiles launched ahead of the rest
        mode = kJoint;
        p.n_global = n_global;
        p.global_row0 = global_first ? 0 : (int32_t)geo.n_tokens;
        p.grid_row0 = global_first ? n_global : 0;
        p.n_dense_rows = n_global;
        p.dense_row0 = p.global_row0;
        p.q_tiles_dense = (n_global + bm - 1) / bm;
        p.n_dense_tiles = batch * heads * p.q_tiles_dense;
    }
    // A launch of few rounds of workgroups over few groups hands its tiles out by list length, longest
    // first (measured at 128x128 tokens in 16x16 groups, 24 heads: +14 % for 3x3 lists, +10 % for 5x5,
    // nothing either way for the equally long criss-cross lists; at 64x64 tokens +7 %).  Larger launches
    // keep the order that lets neighbouring groups share their K/V in the L2.
    p.longest_first = is16(dtype) && geo.num_groups <= 64 && total <= 16 * 256;
    p.fd_tiles_per_rank = make_fastdiv((uint32_t)(batch * heads * p.q_tiles));
    fill_fastdivs(p);
    const hipError_t e = is16(dtype)
                             ? launch_attn_bf16(p, mode, dtype == GRAT_F16, head_dim, (hipStream_t)hip_stream)
                             : launch_attn_f32(p, head_dim, false, (hipStream_t)hip_stream);
    return e == hipSuccess ? GRAT_OK : GRAT_ERR_HIP;
}

extern "C" grat_status grat_attention_fwd(const void* Q, const void* K, const void* V, void* O,
                                          grat_dtype dtype, int32_t batch, int32_t heads,
                                          int32_t head_dim, int64_t stride_b, int64_t stride_h,
                                          int64_t stride_n, float scale, int32_t ndim,
                                          const int32_t* grid, const int32_t* group,
                                          const int32_t* d_kv_count, const int32_t* d_kv_index,
                                          int32_t max_kv, void* hip_stream) {
    return attention_fwd(Q, K, V, O, dtype, batch, heads, head_dim, stride_b, stride_h, stride_n,
                         OutStrides{stride_b, stride_h, stride_n}, scale, 0, 1, ndim, grid, group,
                         d_kv_count, d_kv_index, max_kv, hip_stream);
}

extern "C" grat_status grat_attention_global_fwd(const void* Q, const void* K, const void* V, void* O,
                                                 grat_dtype dtype, int32_t batch, int32_t heads,
                                                 int32_t head_dim, int64_t stride_b, int64_t stride_h,
                                                 int64_t stride_n, float scale, int32_t n_global,
                                                 int32_t global_first, int32_t ndim,
                                                 const int32_t* grid, const int32_t* group,
                                                 const int32_t* d_kv_count, const int32_t* d_kv_index,
                                                 int32_t max_kv, void* hip_stream) {
    return attention_fwd(Q, K, V, O, dtype, batch, heads, head_dim, stride_b, stride_h, stride_n,
                         OutStrides{stride_b, stride_h, stride_n}, scale, n_global, global_first,
                         ndim, grid, group, d_kv_count, d_kv_index, max_kv, hip_stream);
}

extern "C" grat_status grat_attention_packed_fwd(const void* QKV, void* O, grat_dtype dtype,
                                                 int32_t batch, int32_t heads, int32_t head_dim,
                                                 float scale, int32_t n_global, int32_t global_first,
                                                 int32_t ndim, const int32_t* grid, const int32_t* group,
                                                 const int32_t* d_kv_count, const int32_t* d_kv_index,
                                                 int32_t max_kv, void* hip_stream) {
    if (!QKV || !O) return GRAT_ERR_NULL;
    if (batch < 1 || heads < 1 || head_dim < 1) return GRAT_ERR_BAD_DIMS;
    if (!is16(dtype) && dtype != GRAT_F32) return GRAT_ERR_UNSUPPORTED;
    Geometry geo;
    const grat_status st = make_geometry(ndim, grid, group, &geo);
    if (st != GRAT_OK) return st;
    if (n_global < 0) return GRAT_ERR_BAD_DIMS;
    const int64_t seq_len = geo.n_tokens + n_global;
    const int64_t hd = (int64_t)heads * head_dim;            // one of Q, K, V of one token
    const size_t esize = is16(dtype) ? 2 : 4;
    const char* base = (const char*)QKV;
    return attention_fwd(base, base + hd * esize, base + 2 * hd * esize, O, dtype, batch, heads,
                         head_dim, seq_len * 3 * hd, head_dim, 3 * hd,
                         OutStrides{seq_len * hd, head_dim, hd}, scale, n_global, global_first, ndim,
                         grid, group, d_kv_count, d_kv_index, max_kv, hip_stream);
}

extern "C" grat_status grat_dense_attention_fwd(const void* Q, const void* K, const void* V, void* O,
                                                grat_dtype dtype, int32_t batch, int32_t heads,
                                                int64_t n_tokens, int32_t head_dim,
                                                int64_t stride_b, int64_t stride_h,
                                                int64_t stride_n, float scale, void* hip_stream) {
    if (n_tokens >= kMaxElems) return GRAT_ERR_BAD_DIMS;
    grat_status st = check_tensors(Q, K, V, O, dtype, batch, heads, head_dim, n_tokens, stride_b,
                                   stride_h, stride_n, scale);
    if (st != GRAT_OK) return st;

    AttnParams p{};
    p.Q = Q; p.K = K; p.V = V; p.O = O;
    p.stride_b = stride_b; p.stride_h = stride_h; p.stride_n = (int32_t)stride_n;
    p.o_stride_b = stride_b; p.o_stride_h = stride_h; p.o_stride_n = (int32_t)stride_n;
    p.batch = batch; p.heads = heads;
    p.scale_log2 = scale * 1.4426950408889634f;
    p.n_tokens = (int32_t)n_tokens;
    const int bm = is16(dtype) ? 256 : 64;
    p.q_tiles = (int32_t)((n_tokens + bm - 1) / bm);
    p.q_tiles_dense = p.q_tiles;
    p.n_dense_rows = (int32_t)n_tokens;
    p.dense_row0 = 0;
    const int64_t total = (int64_t)batch * heads * p.q_tiles;
    if ((int64_t)batch * heads * ((int64_t)p.q_tiles + 8) >= kMaxElems - 8) return GRAT_ERR_UNSUPPORTED;
    p.total_tiles = (int32_t)total;

    fill_fastdivs(p);
    const hipError_t e = is16(dtype)
                             ? launch_attn_bf16(p, kDense, dtype == GRAT_F16, head_dim, (hipStream_t)hip_stream)
                             : launch_attn_f32(p, head_dim, true, (hipStream_t)hip_stream);
    return e == hipSuccess ? GRAT_OK : GRAT_ERR_HIP;
}

extern "C" const char* grat_status_string(grat_status status) {
    switch (status) {
        case GRAT_OK: return "ok";
        case GRAT_ERR_NULL: return "a required pointer is NULL";
        case GRAT_ERR_BAD_DIMS: return "bad dimensions, radius, strides or scale";
        case GRAT_ERR_INDIVISIBLE: return "a group dim does not divide its grid dim";
        case GRAT_ERR_BAD_PATTERN: return "unknown pattern";
        case GRAT_ERR_BUFFER_TOO_SMALL: return "max_kv is smaller than the longest list";
        case GRAT_ERR_UNSUPPORTED: return "shape, dtype, alignment or size not supported";
        case GRAT_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}
