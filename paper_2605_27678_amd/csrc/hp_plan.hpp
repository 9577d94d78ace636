// Internal: host-side plan of the boundary layout transform.
#pragma once
#include <cstdint>
#include <vector>

#include "hp.h"

namespace hp {

// One workgroup's share of a launch: a byte range that is contiguous in the
// source buffer and either contiguous (pitch_rows == 1) or row-strided in the
// destination buffer(s).  32 bytes, read with scalar loads.
struct alignas(16) Tile {
    uint64_t src_off;     // bytes from the base of the source buffer
    uint64_t dst_off;     // bytes from the base of each destination copy
    uint32_t nbytes;      // payload bytes; whole rows when pitch_rows != 1
    uint32_t pitch_rows;  // destination row pitch in rows (1 = dense)
    uint16_t src_buf;     // source buffer index of copy tp = 0
    uint16_t dst_buf0;    // first destination buffer index
    uint32_t reserved;
};
static_assert(sizeof(Tile) == 32, "tile table entry must stay 32 bytes");

struct Options {
    int64_t tile_bytes = 8192;
    int64_t block_threads_fwd = 256;
    int64_t block_threads_bwd = 256;
    int64_t waves_per_cu_fwd = 8;   // 0 = no cap
    int64_t waves_per_cu_bwd = 12;
    int64_t nontemporal_fwd = 2;  // bit 0: streaming loads, bit 1: streaming stores
    int64_t nontemporal_bwd = 3;
};
Options &options();

}  // namespace hp

struct hp_plan {
    hp_layout_t src{}, dst{};
    int32_t batch = 0, seq = 0, hidden = 0, dtype = 0;
    int32_t elem_bytes = 2;
    int64_t row_bytes = 0;
    int64_t n_rows = 0;
    int32_t n_src_bufs = 0, n_dst_bufs = 0;
    int32_t src_copies = 1, dst_copies = 1;
    int64_t dst_rows_per_buf = 0;
    std::vector<int64_t> src_rows;        // per source buffer
    std::vector<hp_segment_t> segments;
    std::vector<hp::Tile> tiles;
    // device side
    hp::Tile *d_tiles = nullptr;
    int device = -1;
};

namespace hp {
// Validates and fills everything except the device fields.  Returns HP_OK or a
// negative error; *plan is only meaningful on HP_OK.
int build_host_plan(const hp_layout_t *src, const hp_layout_t *dst,
                    const hp_token_map_t *map, hp_plan *plan);
}  // namespace hp
