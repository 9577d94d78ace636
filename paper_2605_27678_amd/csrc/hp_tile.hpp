// Internal: what a kernel launch knows about the plan, and how a workgroup finds
// its tile.  Shared by the gfx950 kernels and by a host-side test that walks
// every tile of every launch shape on the CPU (same code, so the index
// arithmetic the GPU runs is checked for bounds without a GPU).
#pragma once
#include <algorithm>
#include <cstddef>
#include <cstdint>

#include "hp_plan.hpp"

#if defined(__HIPCC__)
#define HP_HD __host__ __device__ __forceinline__
#else
#define HP_HD inline
#endif

namespace hp {

// Everything else a kernel needs, also by value.
struct KParams {
    const Seg *segs;            // segment descriptors
    const uint32_t *tree;       // search trees (64-byte aligned nodes of 16 keys)
    uint32_t n_levels;          // levels of this launch's tree
    uint32_t level_off[kMaxTreeLevels];   // start of each level, in keys; level 0 = leaves
    uint32_t tile_bytes;
    uint32_t row_bytes;
    uint32_t rows_per_tile;     // row-strided segments, rows shorter than a tile: tile_bytes / row_bytes
    uint32_t parts_per_row;     // row-strided segments, rows of at least a tile: ceil(row_bytes / tile_bytes); else 0
    uint32_t dst_base;          // index of the first destination pointer in BufTable
    uint32_t dst_copies;        // replicas of each row on the destination side
};

// One workgroup's share of the launch.
struct TileView {
    uint64_t src_off, dst_off;  // bytes from the buffer bases
    uint32_t nbytes;
    uint32_t pitch_rows;        // 1 = dense destination
    uint32_t src_buf, dst_buf0;
    uint32_t src_copies;        // identical TP copies of the source rank
};

// One node of the search tree: 16 ascending keys (padding = UINT32_MAX) fetched
// with one 64-byte scalar load (the tree must sit at a 64-byte aligned address).  Returns how many keys are <= tile, and the
// largest of them.
HP_HD void search_node(const uint32_t *node, uint32_t tile, uint32_t &count, uint32_t &key) {
    const uint32_t *p = (const uint32_t *)__builtin_assume_aligned(node, 64);
    uint32_t c = 0, best = 0;
#pragma unroll
    for (int j = 0; j < kTreeFanout; ++j) {
        const uint32_t v = p[j];
        const bool le = v <= tile;
        c += le ? 1u : 0u;
        best = le ? v : best;
    }
    count = c;
    key = best;
}

// Scalar code: every value here is uniform over the workgroup.  One dependent
// scalar load per tree level, then the descriptor, then the buffer pointers.
HP_HD TileView locate_tile(const KParams &k, uint32_t tile) {
    uint32_t lo = 0, first = 0;
#pragma unroll
    for (int l = kMaxTreeLevels - 1; l >= 0; --l) {
        if ((uint32_t)l < k.n_levels) {
            uint32_t count;
            search_node(k.tree + k.level_off[l] + (size_t)lo * kTreeFanout, tile, count, first);
            lo = lo * kTreeFanout + count - 1;
        }
    }
    const Seg s = k.segs[lo];
    const uint32_t t = tile - first;
    TileView v;
    v.pitch_rows = s.pitch_rows;
    v.src_buf = s.src_buf;
    v.dst_buf0 = s.dst_buf0;
    v.src_copies = s.src_copies;
    if (s.pitch_rows == 1) {
        const uint64_t off = (uint64_t)t * k.tile_bytes;
        const uint64_t left = (uint64_t)s.n_rows * k.row_bytes - off;
        v.src_off = s.src_off + off;
        v.dst_off = s.dst_off + off;
        v.nbytes = left < k.tile_bytes ? (uint32_t)left : k.tile_bytes;
    } else if (k.parts_per_row) {
        // a piece of one row: dense on both sides, handled like a dense tile
        const uint32_t row = t / k.parts_per_row;
        const uint32_t off = (t - row * k.parts_per_row) * k.tile_bytes;
        const uint32_t left = k.row_bytes - off;
        v.pitch_rows = 1;
        v.src_off = s.src_off + (uint64_t)row * k.row_bytes + off;
        v.dst_off = s.dst_off + (uint64_t)row * s.pitch_rows * k.row_bytes + off;
        v.nbytes = left < k.tile_bytes ? left : k.tile_bytes;
    } else {
        const uint64_t row0 = (uint64_t)t * k.rows_per_tile;
        const uint64_t rows_left = s.n_rows - row0;
        const uint32_t rows = rows_left < k.rows_per_tile ? (uint32_t)rows_left : k.rows_per_tile;
        v.src_off = s.src_off + row0 * k.row_bytes;
        v.dst_off = s.dst_off + row0 * s.pitch_rows * k.row_bytes;
        v.nbytes = rows * k.row_bytes;
    }
    return v;
}


// The kernel parameters of a launch with tiles of 1 KiB << variant; segs and
// tree point at the plan's tables wherever the caller keeps them (device memory
// for a launch, the plan's host vectors for the host-side walk).
inline KParams kernel_params(const hp_plan &p, int variant, const Seg *segs, const uint32_t *tree) {
    KParams k;
    k.segs = segs;
    k.tree = tree;
    k.n_levels = p.tree_info[variant].n_levels;
    for (int l = 0; l < kMaxTreeLevels; ++l) k.level_off[l] = p.tree_info[variant].level_off[l];
    k.tile_bytes = tile_bytes_of(variant);
    k.row_bytes = (uint32_t)p.row_bytes;
    k.rows_per_tile = std::max<uint32_t>(1u, k.tile_bytes / k.row_bytes);
    k.parts_per_row = k.row_bytes >= k.tile_bytes ? (k.row_bytes + k.tile_bytes - 1) / k.tile_bytes : 0u;
    k.dst_base = (uint32_t)p.n_src_bufs;
    k.dst_copies = (uint32_t)p.dst_copies;
    return k;
}

}  // namespace hp
