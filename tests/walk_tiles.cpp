// Host-side walk of every tile of every launch shape, with the code the GPU
// runs (hp_tile.hpp): built by tests/test_plan_host.py with ASan + UBSan.
// For random plans and each of the seven tile sizes it checks that
//   - the tiles of a launch partition the segments exactly: every byte of every
//     segment's source range is covered once, in order, by tiles that name the
//     segment's buffers,
//   - every tile stays inside the source buffer and the destination buffers
//     (dense tiles: one byte range; row-strided tiles: whole rows at the pitch),
//   - no tile is empty or larger than the tile size, and lane chunks divide it.
// usage: walk_tiles <seed> <plans>
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "hp_tile.hpp"

#define CHECK(c)                                                                          \
    do {                                                                                  \
        if (!(c)) { std::printf("plan %d variant %d tile %u: %s\n", it, v, t, #c); return 1; } \
    } while (0)

int main(int argc, char **argv) {
    std::mt19937_64 rng(argc > 1 ? std::atoll(argv[1]) : 1);
    const int plans = argc > 2 ? std::atoi(argv[2]) : 300;
    auto R = [&](int lo, int hi) { return (int)(lo + rng() % (uint64_t)(hi - lo + 1)); };
    long tiles_walked = 0;
    int done = 0;
    for (int it = 0; done < plans && it < 100 * plans; ++it) {
        const int cps[] = {1, 2, 4, 8};
        hp_layout_t src{R(1, 3), 1, R(1, 9), 1, 0, 0, 0, 0};
        hp_layout_t dst{R(1, 9), cps[R(0, 3)], R(1, 2), 1, 0, R(0, 1), R(0, 1), R(0, 1)};
        const int batch = dst.dp * R(1, 3), seq = 2 * dst.cp * dst.tp * R(1, 40);
        const int hiddens[] = {1, 3, 8, 24, 72, 520, 1024, 3000, 5120};
        const int hidden = hiddens[R(0, 8)];
        const int n_maps = R(1, 2);
        std::vector<hp_token_map_t> maps(n_maps);
        std::vector<std::vector<int32_t>> store;
        store.reserve(n_maps * 3);
        for (auto &m : maps) {
            std::vector<int32_t> smp, st, ln;
            for (int b = 0; b < batch; ++b) {
                int pos = R(0, 6);
                while (pos < seq && (int)st.size() < 60) {
                    const int len = std::min(seq - pos, R(1, 1 + seq / 3));
                    smp.push_back(b); st.push_back(pos); ln.push_back(len);
                    pos += len + R(0, 9);
                }
            }
            store.push_back(smp); const int32_t *ps = store.back().data();
            store.push_back(st);  const int32_t *pt = store.back().data();
            store.push_back(ln);  const int32_t *pl = store.back().data();
            m = hp_token_map_t{batch, seq, hidden, R(0, 1), (int32_t)smp.size(), ps, pt, pl, nullptr};
        }
        for (auto &m : maps) m.dtype = maps[0].dtype;
        hp_plan p;
        if (hp::build_host_plan(&src, 1, &dst, maps.data(), n_maps, &p) != HP_OK) continue;
        ++done;
        // the device descriptors say what the public segments say (no field narrowed)
        {
            int v = -1; uint32_t t = 0;
            CHECK(p.dsegs.size() == p.segments.size());
            for (size_t i = 0; i < p.segments.size(); ++i) {
                t = (uint32_t)i;
                CHECK((int64_t)p.dsegs[i].n_rows == p.segments[i].n_rows);
                CHECK((int64_t)p.dsegs[i].pitch_rows == p.segments[i].dst_row_stride);
                CHECK((int32_t)p.dsegs[i].src_buf == p.segments[i].src_buf);
                CHECK((int32_t)p.dsegs[i].dst_buf0 == p.segments[i].dst_buf0);
                CHECK(p.dsegs[i].src_off == (uint64_t)p.segments[i].src_row0 * (uint64_t)p.row_bytes);
                CHECK(p.dsegs[i].dst_off == (uint64_t)p.segments[i].dst_row0 * (uint64_t)p.row_bytes);
            }
        }
        // the tree has to be 64-byte aligned, as it is in the device block
        uint32_t *tree = (uint32_t *)std::aligned_alloc(64, (p.tree.size() * 4 + 63) / 64 * 64 + 64);
        std::copy(p.tree.begin(), p.tree.end(), tree);
        const uint64_t row = (uint64_t)p.row_bytes;
        const uint32_t lane = row % 16 == 0 ? 16 : row % 4 == 0 ? 4 : (uint32_t)p.elem_bytes;
        for (int v = 0; v < hp::kTileVariants; ++v) {
            const hp::KParams k = hp::kernel_params(p, v, p.dsegs.data(), tree);
            const uint32_t n_tiles = p.n_tiles(v);
            size_t seg = 0;
            uint64_t covered = 0;                      // bytes of the current segment already seen
            for (uint32_t t = 0; t < n_tiles; ++t) {
                const hp::TileView tv = hp::locate_tile(k, t);
                ++tiles_walked;
                while (seg < p.dsegs.size() && covered == (uint64_t)p.dsegs[seg].n_rows * row) { ++seg; covered = 0; }
                CHECK(seg < p.dsegs.size());
                const hp::Seg &s = p.dsegs[seg];
                CHECK(tv.src_buf == s.src_buf && tv.dst_buf0 == s.dst_buf0 && tv.src_copies == s.src_copies);
                CHECK(tv.nbytes > 0 && tv.nbytes % lane == 0);
                CHECK(tv.src_off == s.src_off + covered);            // in order, no gap, no overlap
                CHECK(tv.src_off + tv.nbytes <= (uint64_t)p.src_rows[s.src_buf] * row);
                CHECK(s.src_buf + s.src_copies <= (uint32_t)p.n_src_bufs);
                CHECK(s.dst_buf0 + k.dst_copies <= (uint32_t)p.n_dst_bufs);
                const uint64_t dst_bytes = (uint64_t)p.dst_rows_per_buf * row;
                if (tv.pitch_rows == 1) {
                    CHECK(tv.nbytes <= k.tile_bytes);
                    const uint64_t r0 = covered / row, in_row = covered % row;
                    const uint64_t want = s.pitch_rows == 1 ? s.dst_off + covered
                                                            : s.dst_off + r0 * s.pitch_rows * row + in_row;
                    CHECK(tv.dst_off == want);
                    if (s.pitch_rows != 1) CHECK(in_row + tv.nbytes <= row);   // a piece never leaves its row
                    CHECK(tv.dst_off + tv.nbytes <= dst_bytes);
                } else {
                    CHECK(tv.nbytes % row == 0 && covered % row == 0 && tv.nbytes <= std::max<uint64_t>(k.tile_bytes, row));
                    CHECK(tv.dst_off == s.dst_off + covered / row * s.pitch_rows * row);
                    const uint64_t rows = tv.nbytes / row;
                    CHECK(tv.dst_off + (rows - 1) * tv.pitch_rows * row + row <= dst_bytes);
                }
                covered += tv.nbytes;
            }
            while (seg < p.dsegs.size() && covered == (uint64_t)p.dsegs[seg].n_rows * row) { ++seg; covered = 0; }
            uint32_t t = n_tiles;
            CHECK(seg == p.dsegs.size() && covered == 0);             // every segment fully covered
        }
        std::free(tree);
    }
    std::printf("plans %d tiles %ld\n", done, tiles_walked);
    return done == plans ? 0 : 2;
}
