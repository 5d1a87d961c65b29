// Element order of the KV cache (private to the library; callers use spec_kv_import/export).
//
// fp32 caches are plain: [layer][slot][k|v][kv head][position][dim].
//
// bf16 caches are laid out for the attention kernel's matrix-instruction operands.  The positions
// are grouped in blocks of 32, and a slot is stored as [layer][slot][block][kv head]: the wavefronts
// that stream the heads of one sequence advance together, so at any moment they read one contiguous
// stretch of memory (n_kv_heads * 64 * hd elements per block) and spread over all memory channels
// whatever the slot capacity is.  (With [kv head][block] the distance between the streams is the
// capacity of a head, and for some capacities -- 129 blocks of 128-dim heads, say -- the streams
// fell on few channels: the attention launch took 14 % longer.)  One head's share of a block holds a
// key part of 32*hd elements followed by a value part of 32*hd elements:
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

// Paged mode keeps the same order inside a 32-position block; only where a block lives changes.
// Element offset of block blk of (layer, slot, head), either mode (bf16).
__host__ __device__ inline size_t cache_block_base(const CacheGeom& g, int layer, int slot, int head, int blk)
{
    if (!g.table) return cache_head_base(g, layer, slot, head) + (size_t)blk * g.blk_stride;
    int page = g.table[(size_t)slot * g.blocks_per_slot + blk];
    if (page < 0) page = 0;   // never for a position the step may touch; keeps a stray access in bounds
    return (size_t)page * g.page_stride + ((size_t)layer * g.n_kv_heads + head) * (64 * g.head_dim);
}

// pages: make sure the blocks covering positions [pos0, pos1) of a slot exist.  Returns false when
// the pool ran dry (nothing is rolled back: the caller flags the sequence).
__device__ inline bool pool_cover(const PagePool& p, int slot, int pos0, int pos1)
{
    if (!p.table || pos1 <= pos0) return true;
    for (int blk = pos0 >> 5; blk <= (pos1 - 1) >> 5; ++blk) {
        int32_t* e = p.table + (size_t)slot * p.blocks_per_slot + blk;
        if (*e >= 0) continue;
        const int idx = atomicSub(p.free_top, 1) - 1;
        if (idx < 0) {
            atomicAdd(p.free_top, 1);
            return false;
        }
        *e = p.free_stack[idx];
    }
    return true;
}

// pages: give back every block of a slot that holds no position below new_len
__device__ inline void pool_trim(const PagePool& p, int slot, int new_len)
{
    if (!p.table) return;
    for (int blk = (new_len + 31) >> 5; blk < p.blocks_per_slot; ++blk) {
        int32_t* e = p.table + (size_t)slot * p.blocks_per_slot + blk;
        if (*e < 0) break;   // blocks are allocated from the front: the first hole ends the run
        p.free_stack[atomicAdd(p.free_top, 1)] = *e;
        *e = -1;
    }
}

// bf16 tiled order inside one block (t32 = position & 31), relative to cache_block_base
__host__ __device__ inline size_t tiled_k_within(int hd, int t32, int dim)
{
    const int sub = t32 >> 4, t16 = t32 & 15;
    return ((size_t)(sub * (hd >> 3) + (dim >> 3)) * 16 + t16) * 8 + (dim & 7);
}

__host__ __device__ inline size_t tiled_v_within(int hd, int t32, int dim)
{
    const int sub = t32 >> 4, t16 = t32 & 15;
    const int g = t16 >> 2, e = (t16 & 3) + 4 * sub;
    return 32 * hd + ((size_t)(dim >> 4) * 64 + g * 16 + (dim & 15)) * 8 + e;
}

// fp32 plain order, offsets relative to cache_head_base (k plane; the v plane is v_plane further)
__host__ __device__ inline size_t plain_offset(const CacheGeom& g, int kv, int pos, int dim)
{
    return (size_t)kv * g.n_kv_heads * g.head_stride + (size_t)pos * g.head_dim + dim;
}

}  // namespace specv
