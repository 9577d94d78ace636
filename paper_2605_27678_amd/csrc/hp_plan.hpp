// Internal: host-side plan of the boundary layout transform.
#pragma once
#include <cstdint>
#include <mutex>
#include <vector>

#include "hp.h"

namespace hp {

// Device-side descriptor of one segment: a run of image-token rows that is
// contiguous in its source buffer and contiguous (pitch_rows == 1) or evenly
// row-strided in each destination copy.  32 bytes; the whole table of a plan is
// a few KB and stays hot in the scalar cache.
struct alignas(16) Seg {
    uint64_t src_off;     // bytes from the base of the source buffer
    uint64_t dst_off;     // bytes from the base of each destination copy
    uint32_t n_rows;      // rows of row_bytes each
    uint32_t pitch_rows;  // destination row pitch in rows (1 = dense)
    uint16_t src_buf;     // source buffer index of copy tp = 0
    uint16_t dst_buf0;    // first destination buffer index
    uint32_t src_copies;  // identical TP copies of the source rank (buffers src_buf .. +src_copies-1)
};
static_assert(sizeof(Seg) == 32, "segment descriptor must stay 32 bytes");
// Longest run one descriptor can describe; the builder starts a new segment
// rather than merging past it.
constexpr uint32_t kMaxSegRows = UINT32_MAX;

// A launch cuts every segment into tiles of 1 KiB << v bytes, one workgroup per
// tile.  For each variant v the plan keeps first_tile[v][s] = number of tiles of
// segments 0..s-1 and, for the device, a 16-ary search tree over those keys, so
// a workgroup finds its segment with one 64-byte scalar load per tree level
// (one level up to 16 segments, two up to 256, ...) out of a tiny,
// cache-resident table instead of reading a per-tile table from HBM.
constexpr int kTileVariants = 7;
constexpr int kTreeFanout = 16;
constexpr int kMaxTreeLevels = 4;          // 16^4 = 65536 segments
inline uint32_t tile_bytes_of(int v) { return 1024u << v; }

// Where one variant's search tree sits in the plan's tree array (in uint32
// elements).  Level 0 holds the keys first_tile[v][0..n), padded with
// UINT32_MAX to whole 16-key nodes; key j of level l+1 is key 16*j of level l.
struct TreeInfo {
    uint32_t n_levels;
    uint32_t level_off[kMaxTreeLevels];
};

// How one direction is launched.  Lives in the plan; seeded from the
// process-wide defaults, overridden by hp_plan_set_launch or hp_plan_tune.
struct Launch {
    int32_t tile_variant;   // tile = 1 KiB << tile_variant
    int32_t block;          // threads per workgroup
    int32_t waves_per_cu;   // resident-wave cap, 0 = none
    int32_t nontemporal;    // bit 0 streaming loads, bit 1 streaming stores
};

struct Options {
    // HP_AUTO (-1) = chosen per plan from its replica counts (see default_launch)
    int64_t tile_bytes_fwd = -1, tile_bytes_bwd = -1;
    int64_t block_threads_fwd = -1, block_threads_bwd = -1;
    int64_t waves_per_cu_fwd = -1, waves_per_cu_bwd = -1;   // 0 = no cap
    int64_t nontemporal_fwd = 2, nontemporal_bwd = 3;       // bit 0 loads, bit 1 stores
};
Options &options();             // guarded by options_mutex()
std::mutex &options_mutex();
int tile_variant_of(int64_t tile_bytes);   // -1 unless 1 KiB << v, v < kTileVariants

}  // namespace hp

struct hp_plan {
    hp_layout_t src{}, dst{};
    int32_t batch = 0, seq = 0, hidden = 0, dtype = 0;
    int32_t n_maps = 1;                   // microbatches folded into this plan
    int32_t n_edges = 1;                  // source modules joined into the one destination
    int32_t elem_bytes = 2;
    int64_t row_bytes = 0;
    int64_t n_rows = 0;
    int32_t n_src_bufs = 0, n_dst_bufs = 0;   // totals over all microbatches
    int32_t src_copies = 1, dst_copies = 1;   // src_copies: of the first edge (edges may differ, see seg_copies)
    int64_t bwd_bytes = 0, bwd_accum_bytes = 0;   // algorithmic bytes of the two backward flavours
    int64_t dst_rows_per_buf = 0;
    std::vector<int64_t> src_rows;        // per source buffer
    std::vector<uint8_t> src_leader;      // per source buffer: 1 = copy tp 0 of its rank (the one forward reads)
    std::vector<int32_t> seg_copies;      // per segment: TP copies of its source rank
    std::vector<hp_segment_t> segments;   // public view (rows)
    std::vector<hp::Seg> dsegs;           // device view (bytes)
    std::vector<uint32_t> first_tile;     // kTileVariants x (n_segments + 1), row-major
    std::vector<uint32_t> tree;           // the search trees of all variants, 64-byte aligned nodes
    hp::TreeInfo tree_info[hp::kTileVariants] = {};
    hp::Launch fwd{}, bwd{}, acc{};       // hp_forward, hp_backward, hp_backward_accumulate
    // device side
    hp::Seg *d_segs = nullptr;
    uint32_t *d_tree = nullptr;
    size_t d_bytes = 0;                   // size of the device block behind d_segs
    int device = -1;
    // Streams on which work that reads the device block has been enqueued (as
    // opaque handles).  hp_plan_destroy orders the reuse of the block after them.
    mutable std::mutex use_mu;
    mutable std::vector<void *> used_streams;

    void note_stream(void *stream) const {
        std::lock_guard<std::mutex> lk(use_mu);
        for (void *s : used_streams)
            if (s == stream) return;
        used_streams.push_back(stream);
    }

    uint32_t n_tiles(int variant) const {
        const size_t n = segments.size();
        return n ? first_tile[(size_t)variant * (n + 1) + n] : 0u;
    }
};

namespace hp {
// Validates and fills everything except the device fields for `n_edges` source
// modules that feed one destination module, each with `n_maps` token maps
// (maps[e * n_maps + m] = edge e, microbatch m; all share batch, sequence length,
// hidden size and dtype, and the spans of different edges must not overlap).
// Source buffers are listed edge by edge, inside an edge microbatch by
// microbatch; destination buffers microbatch by microbatch, shared by all
// edges.  Returns HP_OK or a negative error; *plan is only meaningful on HP_OK.
int build_host_plan(const hp_layout_t *srcs, int32_t n_edges, const hp_layout_t *dst,
                    const hp_token_map_t *maps, int32_t n_maps, hp_plan *plan);
}  // namespace hp
