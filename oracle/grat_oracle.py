"""CPU oracle for GRAT grouped sparse attention (float64, numpy).

TEST INFRASTRUCTURE ONLY.  This is the slow, plain definition of what the GPU library
computes.  It shares no code with the HIP path and must never be imported by it; only the
tests, the smoke check and the benchmark's cpu_baseline leg call it.

What it follows (paper sections / equations, numbered in order of appearance):
  * Sec. 3.1, Eq. 1        softmax(Q K^T * scale) V per head;
  * Sec. 3.2, Eq. 2-4      2D grouping: token (i, j) is in group (i // g1, j // g2);
  * Sec. 3.2, Eq. 5-6      GRAT-B: query group (p, q) attends KV groups (m, n) with
                           |m - p| <= b and |n - q| <= b;
  * Sec. 3.2, Eq. 7-8      GRAT-X: KV groups in the same group-row or the same
                           group-column (the printed "n = p" is read as "n = q", which
                           is what the prose and the printed sparsities say);
  * Sec. 3.2, Eq. 9-11     3D grouping with (t // g1, i // g2, j // g3);
  * Sec. 3.2, Eq. 12-13    3D GRAT-B with per-axis radii (b_t, b_h, b_w);
  * Sec. 3.2, Eq. 14-15    3D GRAT-X.  Printed predicate: at least ONE group coordinate
                           equal (three planes) -> pattern "cross_planes".  The prose of
                           Sec. 3.2 ahead of Eq. 14-15 describes the three axis lines
                           through the group: at least ndim-1 coordinates equal ->
                           pattern "cross".  In 2D the two coincide.

Readings where the paper is silent: neighbours outside the grid are dropped (no wrap, no
window shift); a group attends itself; tokens are stored row-major over the grid (last
dim fastest) and grouping is pure index arithmetic; a grid that a group dim does not
divide gets a ragged last group (floor division in Eq. 2-4); block lists are ascending
in the linear group id ((p0*G1)+p1)*G2+p2 and padded with -1.

The attention mask is always derived from TOKEN COORDINATES (Eq. 2-4 then the set
predicate), never from a block list, so the list enumerator and the mask pin each other.

Pins (tests/test_oracle_*.py): hand-enumerated 4x4 lists (tests/golden), closed-form
list counts, the sparsity and farthest-token figures printed in Tab. 1 / Tab. 3 / Tab. 6,
per-query brute-force loops, full coverage == dense softmax attention (checked against
torch's float64 scaled_dot_product_attention), rows of P sum to 1, constant V passes
through, K == 0 gives the mean of V over the attendable set, group 1x1 == per-token
window / criss-cross attention, and mirror / transpose equivariance.  The joint-sequence
functions (prompt tokens next to the grid) are pinned by per-query loops, by their reduction
to the plain functions for n_global = 0 and on the grid block, and by the printed GRAT-X
sparsities counted from their mask.
"""
from __future__ import annotations

from typing import Optional, Sequence, Tuple

import numpy as np

PATTERNS = ("block", "cross", "cross_planes", "dense")


# ----------------------------------------------------------------------------------------
# Grouping (Eq. 2-4, Eq. 9-11)
# ----------------------------------------------------------------------------------------
def group_grid(grid: Sequence[int], group: Sequence[int]) -> Tuple[int, ...]:
    """Number of groups along each axis; a ragged last group counts (floor division)."""
    assert len(grid) == len(group) and len(grid) >= 1
    assert all(t >= 1 for t in grid) and all(g >= 1 for g in group)
    return tuple((t + g - 1) // g for t, g in zip(grid, group))


def token_coords(rows: np.ndarray, grid: Sequence[int]) -> np.ndarray:
    """Token row index -> grid coordinates, row-major with the last dim fastest. [R, ndim]"""
    return np.stack(np.unravel_index(np.asarray(rows, dtype=np.int64), tuple(grid)), axis=-1)


def token_group_coords(rows: np.ndarray, grid: Sequence[int], group: Sequence[int]) -> np.ndarray:
    """Group coordinates p_k = x_k // g_k of each token. [R, ndim]"""
    return token_coords(rows, grid) // np.asarray(group, dtype=np.int64)


# ----------------------------------------------------------------------------------------
# Attendable-set predicate on group coordinates (Eq. 5-8, Eq. 12-15)
# ----------------------------------------------------------------------------------------
def attendable(pq: np.ndarray, pk: np.ndarray, pattern: str, radius: Sequence[int]) -> np.ndarray:
    """True where the KV group at coords pk is attendable from the query group at pq.

    pq, pk broadcast against each other over leading dims; the last dim is ndim.
    """
    assert pattern in PATTERNS, pattern
    pq = np.asarray(pq, dtype=np.int64)
    pk = np.asarray(pk, dtype=np.int64)
    ndim = pq.shape[-1]
    if pattern == "dense":
        return np.ones(np.broadcast_shapes(pq.shape, pk.shape)[:-1], dtype=bool)
    if pattern == "block":
        b = np.asarray(radius, dtype=np.int64)
        assert b.shape == (ndim,) and (b >= 0).all()
        return (np.abs(pk - pq) <= b).all(axis=-1)
    n_equal = (pk == pq).sum(axis=-1)
    if pattern == "cross":
        return n_equal >= ndim - 1
    return n_equal >= 1  # cross_planes


def block_lists(grid: Sequence[int], group: Sequence[int], pattern: str,
                radius: Sequence[int]) -> Tuple[np.ndarray, np.ndarray]:
    """Per query group: the ascending list of attendable KV group ids.

    Returns (kv_count int32 [G], kv_index int32 [G, max_kv] padded with -1) where max_kv is
    the longest list.
    """
    gg = group_grid(grid, group)
    G = int(np.prod(gg))
    coords = np.stack(np.unravel_index(np.arange(G), gg), axis=-1)  # [G, ndim]
    lists = []
    for gamma in range(G):
        ok = attendable(coords[gamma], coords, pattern, radius)
        lists.append(np.nonzero(ok)[0])
    count = np.array([len(l) for l in lists], dtype=np.int32)
    assert (count >= 1).all()
    index = np.full((G, int(count.max())), -1, dtype=np.int32)
    for gamma, l in enumerate(lists):
        index[gamma, :len(l)] = l
    return count, index


def mask_rows(rows: np.ndarray, grid: Sequence[int], group: Sequence[int], pattern: str,
              radius: Sequence[int]) -> np.ndarray:
    """Boolean [R, N]: may query token rows[r] attend KV token j?  From token coordinates."""
    N = int(np.prod(grid))
    pk = token_group_coords(np.arange(N), grid, group)          # [N, ndim]
    pq = token_group_coords(np.asarray(rows), grid, group)      # [R, ndim]
    return attendable(pq[:, None, :], pk[None, :, :], pattern, radius)


def attended_pairs(grid: Sequence[int], group: Sequence[int], pattern: str,
                   radius: Sequence[int]) -> int:
    """Number of (query token, KV token) pairs the pattern keeps, per head."""
    gg = group_grid(grid, group)
    # tokens in each group (ragged last groups are smaller)
    sizes = np.ones(gg, dtype=np.int64)
    for k, (t, g, n) in enumerate(zip(grid, group, gg)):
        ext = np.minimum(g, t - np.arange(n) * g)
        shape = [1] * len(gg)
        shape[k] = n
        sizes = sizes * ext.reshape(shape)
    sizes = sizes.reshape(-1)
    count, index = block_lists(grid, group, pattern, radius)
    total = 0
    for gamma in range(len(count)):
        total += int(sizes[gamma]) * int(sizes[index[gamma, :count[gamma]]].sum())
    return total


# ----------------------------------------------------------------------------------------
# Attention (Eq. 1 restricted to the attendable set)
# ----------------------------------------------------------------------------------------
def decode_bf16(bits: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 bit patterns -> float64 (exact)."""
    assert bits.dtype == np.uint16
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def as_f64(x: np.ndarray) -> np.ndarray:
    """Inputs arrive as float16/float32/float64 values or as uint16 bf16 bit patterns."""
    return decode_bf16(x) if x.dtype == np.uint16 else np.asarray(x, dtype=np.float64)


def masked_softmax_rows(S: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """Row softmax of S over the True entries of mask; False entries get weight 0."""
    assert mask.any(axis=-1).all(), "a query row with an empty attendable set"
    S = np.where(mask, S, -np.inf)
    S = S - S.max(axis=-1, keepdims=True)
    P = np.exp(S)
    return P / P.sum(axis=-1, keepdims=True)


def masked_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, mask: np.ndarray,
                     scale: float, return_weights: bool = False):
    """One head.  q [R, d], k [N, d], v [N, d], mask [R, N] -> [R, d] (float64)."""
    q, k, v = as_f64(q), as_f64(k), as_f64(v)
    P = masked_softmax_rows((q @ k.T) * float(scale), mask)
    O = P @ v
    return (O, P) if return_weights else O


def grat_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, grid: Sequence[int],
                   group: Sequence[int], pattern: str, radius: Sequence[int], scale: float,
                   row_chunk: int = 1024) -> np.ndarray:
    """All rows.  Q, K, V [B, H, N, d] -> O float64 [B, H, N, d]."""
    B, H, N, d = Q.shape
    assert N == int(np.prod(grid))
    O = np.empty((B, H, N, d), dtype=np.float64)
    for r0 in range(0, N, row_chunk):
        rows = np.arange(r0, min(N, r0 + row_chunk))
        mask = mask_rows(rows, grid, group, pattern, radius)
        for b in range(B):
            for h in range(H):
                O[b, h, rows] = masked_attention(Q[b, h, rows], K[b, h], V[b, h], mask, scale)
    return O


def grat_attention_rows(Q: np.ndarray, K: np.ndarray, V: np.ndarray, samples: np.ndarray,
                        grid: Sequence[int], group: Sequence[int], pattern: str,
                        radius: Sequence[int], scale: float) -> np.ndarray:
    """Selected rows only.  samples int [R, 3] of (batch, head, token row) -> O float64 [R, d].

    Only the attendable keys of each sampled row are touched, so this stays cheap on the
    large workloads.
    """
    samples = np.asarray(samples, dtype=np.int64)
    d = Q.shape[-1]
    out = np.empty((len(samples), d), dtype=np.float64)
    N = int(np.prod(grid))
    pk = token_group_coords(np.arange(N), grid, group)
    for i, (b, h, r) in enumerate(samples):
        pq = token_group_coords(np.array([r]), grid, group)[0]
        keys = np.nonzero(attendable(pq, pk, pattern, radius))[0]
        q = as_f64(Q[b, h, r])
        s = (as_f64(K[b, h, keys]) @ q) * float(scale)
        p = np.exp(s - s.max())
        p /= p.sum()
        out[i] = p @ as_f64(V[b, h, keys])
    return out


# ----------------------------------------------------------------------------------------
# Joint sequences: prompt ("global") tokens next to the grid tokens
# ----------------------------------------------------------------------------------------
# The method section defines attention over the spatial tokens only; the models it is applied to
# attend over a joint sequence of prompt tokens and image / video tokens, and the FLOPs
# sparsities printed for GRAT-X in the ablation table are reproduced only if every image query
# also attends 512 prompt tokens.  Reading taken here: n_global prompt tokens are stored before
# (global_first) or after the grid tokens; a grid query attends its attendable groups plus all
# prompt tokens; a prompt query attends every token.
def joint_mask_rows(rows: np.ndarray, n_global: int, global_first: bool, grid: Sequence[int],
                    group: Sequence[int], pattern: str, radius: Sequence[int]) -> np.ndarray:
    """Boolean [R, n_global + N]: may query row rows[r] of the joint sequence attend row j?"""
    N = int(np.prod(grid))
    rows = np.asarray(rows, dtype=np.int64)
    g0 = 0 if global_first else N              # first prompt row
    s0 = n_global if global_first else 0       # first grid row
    is_global_q = (rows >= g0) & (rows < g0 + n_global)
    mask = np.zeros((len(rows), n_global + N), dtype=bool)
    mask[:, g0:g0 + n_global] = True           # everyone attends the prompt tokens
    mask[is_global_q, :] = True                # prompt queries attend everything
    grid_q = np.nonzero(~is_global_q)[0]
    if len(grid_q):
        mask[np.ix_(grid_q, np.arange(s0, s0 + N))] = mask_rows(rows[grid_q] - s0, grid, group, pattern, radius)
    return mask


def joint_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, n_global: int, global_first: bool,
                    grid: Sequence[int], group: Sequence[int], pattern: str, radius: Sequence[int],
                    scale: float, row_chunk: int = 512) -> np.ndarray:
    """All rows of the joint sequence.  Q, K, V [B, H, n_global + N, d] -> O float64."""
    B, H, L, d = Q.shape
    assert L == n_global + int(np.prod(grid))
    O = np.empty((B, H, L, d), dtype=np.float64)
    for r0 in range(0, L, row_chunk):
        rows = np.arange(r0, min(L, r0 + row_chunk))
        mask = joint_mask_rows(rows, n_global, global_first, grid, group, pattern, radius)
        for b in range(B):
            for h in range(H):
                O[b, h, rows] = masked_attention(Q[b, h, rows], K[b, h], V[b, h], mask, scale)
    return O


def joint_attention_rows(Q, K, V, samples: np.ndarray, n_global: int, global_first: bool,
                         grid: Sequence[int], group: Sequence[int], pattern: str,
                         radius: Sequence[int], scale: float) -> np.ndarray:
    """Selected (batch, head, row) triples of the joint sequence -> O float64 [R, d]."""
    samples = np.asarray(samples, dtype=np.int64)
    out = np.empty((len(samples), Q.shape[-1]), dtype=np.float64)
    for i, (b, h, r) in enumerate(samples):
        keys = np.nonzero(joint_mask_rows(np.array([r]), n_global, global_first, grid, group, pattern, radius)[0])[0]
        s = (as_f64(K[b, h, keys]) @ as_f64(Q[b, h, r])) * float(scale)
        p = np.exp(s - s.max())
        out[i] = (p / p.sum()) @ as_f64(V[b, h, keys])
    return out


def dense_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float,
                    row_chunk: int = 1024) -> np.ndarray:
    """Eq. 1 with no restriction.  Q [B, H, Nq, d], K, V [B, H, Nk, d] -> float64 O."""
    B, H, Nq, d = Q.shape
    O = np.empty((B, H, Nq, d), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            k, v = as_f64(K[b, h]), as_f64(V[b, h])
            for r0 in range(0, Nq, row_chunk):
                q = as_f64(Q[b, h, r0:r0 + row_chunk])
                S = (q @ k.T) * float(scale)
                S -= S.max(axis=-1, keepdims=True)
                P = np.exp(S)
                O[b, h, r0:r0 + row_chunk] = (P / P.sum(axis=-1, keepdims=True)) @ v
    return O


def dense_attention_rows(Q, K, V, samples: np.ndarray, scale: float) -> np.ndarray:
    samples = np.asarray(samples, dtype=np.int64)
    out = np.empty((len(samples), Q.shape[-1]), dtype=np.float64)
    cache = {}
    for i, (b, h, r) in enumerate(samples):
        if (b, h) not in cache:
            cache.clear()
            cache[(b, h)] = (as_f64(K[b, h]), as_f64(V[b, h]))
        k, v = cache[(b, h)]
        s = (k @ as_f64(Q[b, h, r])) * float(scale)
        p = np.exp(s - s.max())
        out[i] = (p / p.sum()) @ v
    return out
