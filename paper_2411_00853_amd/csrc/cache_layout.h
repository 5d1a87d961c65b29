// Element order of the KV cache (private to the library; callers use spec_kv_import/export).
//
// fp32 caches are plain: [layer][slot][k|v][kv head][position][dim].
//
// bf16 caches are laid out for the attention kernel's matrix-instruction operands.  Per (layer,
// slot, kv head) the positions are grouped in blocks of 32; a block holds a key part of 32*hd
// elements followed by a value part of 32*hd elements:
//   key part:   [sub = 2 halves of 16 positions][dim group = hd/8][position in half = 16][8 dims]
//               -> the A operand of S^T = K * Q^T for one half and one 32-dim step is a contiguous
//                  1 KiB run: lane l reads 16 bytes at dim group 4*step + l/16, position l%16.
//   value part: [dim tile = hd/16][lane = 64][8 positions], lane = 16*g + n holds dim 16*tile + n
//               at positions {4g..4g+3} of the first half then {4g..4g+3} of the second half
//               -> the A operand of O^T = V^T * P^T is a contiguous 1 KiB run per dim tile, and its
//                  position order matches the registers in which the score instruction leaves P^T.
#pragma once

#include "common.h"

namespace specv {

__host__ __device__ inline size_t cache_head_base(const CacheGeom& g, int layer, int slot, int head)
{
    return (size_t)layer * g.layer_stride + (size_t)slot * g.slot_stride + (size_t)head * g.head_stride;
}

// bf16 tiled order, offsets relative to cache_head_base
__host__ __device__ inline size_t tiled_k_offset(int hd, int pos, int dim)
{
    const int blk = pos >> 5, t32 = pos & 31, sub = t32 >> 4, t16 = t32 & 15;
    return (size_t)blk * (64 * hd) + ((size_t)(sub * (hd >> 3) + (dim >> 3)) * 16 + t16) * 8 + (dim & 7);
}

__host__ __device__ inline size_t tiled_v_offset(int hd, int pos, int dim)
{
    const int blk = pos >> 5, t32 = pos & 31, sub = t32 >> 4, t16 = t32 & 15;
    const int g = t16 >> 2, e = (t16 & 3) + 4 * sub;
    return (size_t)blk * (64 * hd) + 32 * hd + ((size_t)(dim >> 4) * 64 + g * 16 + (dim & 15)) * 8 + e;
}

// fp32 plain order, offsets relative to cache_head_base (k plane; the v plane is v_plane further)
__host__ __device__ inline size_t plain_offset(const CacheGeom& g, int kv, int pos, int dim)
{
    return (size_t)kv * g.n_kv_heads * g.head_stride + (size_t)pos * g.head_dim + dim;
}

}  // namespace specv
