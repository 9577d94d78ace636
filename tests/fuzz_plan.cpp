// Host-only fuzz of the plan builder, built with AddressSanitizer and UBSan by
// tests/test_plan_host.py: random grids and token maps (one case in ten may be
// invalid anywhere), joined and batched; every accepted plan's segments must lie
// inside the buffers the plan reports.  usage: fuzz_plan <seed> <iterations>
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>
#include "hp_plan.hpp"
int main(int argc, char **argv) {
    std::mt19937_64 rng(argc > 1 ? atoll(argv[1]) : 1);
    auto R = [&](int lo, int hi) { return (int)(lo + rng() % (uint64_t)(hi - lo + 1)); };
    long ok = 0, bad = 0;
    const int iterations = argc > 2 ? atoi(argv[2]) : 20000;
    for (int it = 0; it < iterations; ++it) {
        int n_edges = R(1, 3), n_maps = R(1, 3);
        std::vector<hp_layout_t> srcs(n_edges);
        const bool wild = R(0, 9) == 0;                       // one case in ten may be invalid anywhere
        for (auto &s : srcs) s = hp_layout_t{R(wild ? 0 : 1, 4), 1 + (wild && R(0, 5) == 0), R(wild ? 0 : 1, 9), R(1, 2), R(wild ? -1 : 0, 5), wild && R(0, 5) == 0, 0, 0};
        const int cps[] = {1, 2, 4, 8};
        hp_layout_t dst{R(wild ? 0 : 1, wild ? 17 : 6), cps[R(0, 3)], R(1, 2), 1, R(0, 3), R(0, 1), R(0, 1), R(0, 1)};
        int batch = dst.dp * R(1, 3), seq = 2 * dst.cp * dst.tp * R(1, 6), hidden = R(wild ? 0 : 1, 40);
        if (wild && R(0, 3) == 0) { batch = R(0, 6); seq = R(0, 96); }
        std::vector<hp_token_map_t> maps(n_edges * n_maps);
        std::vector<std::vector<int32_t>> store;
        store.reserve(maps.size() * 4);
        for (auto &m : maps) {
            int k = R(0, 6);
            std::vector<int32_t> smp(k), st(k), ln(k), dp(k);
            int b = 0, pos = 0;
            for (int i = 0; i < k; ++i) {
                if (R(0, 3) == 0) { ++b; pos = 0; }
                if (wild && R(0, 10) == 0) b = R(-1, 7);
                if (b >= batch && !wild) b = batch - 1;
                smp[i] = b;
                pos += R(0, 5) - (wild && R(0, 8) == 0 ? 3 : 0);
                st[i] = pos;
                ln[i] = R(1, 12) + (wild && R(0, 10) == 0 ? -3 : 0);
                pos += ln[i];
                dp[i] = R(0, 9);   // reduced below to the edge's dp
            }
            std::sort(dp.begin(), dp.end());
            if (wild && R(0, 5) == 0 && k > 1) std::swap(dp[0], dp[k - 1]);
            store.push_back(smp); const int32_t *ps = store.back().data();
            store.push_back(st);  const int32_t *pt = store.back().data();
            store.push_back(ln);  const int32_t *pl = store.back().data();
            store.push_back(dp);  const int32_t *pd = store.back().data();
            m = hp_token_map_t{batch, seq, hidden, wild && R(0, 9) == 0 ? 2 : 0, k, ps, pt, pl, nullptr};
            if (wild && R(0, 20) == 0) m.hidden += 1;
        }
        hp_plan p;
        int rc = hp::build_host_plan(srcs.data(), n_edges, &dst, maps.data(), n_maps, &p);
        if (rc == HP_OK) {
            ++ok;
            // every segment must stay inside its buffers
            for (size_t i = 0; i < p.segments.size(); ++i) {
                const hp_segment_t &s = p.segments[i];
                if (s.src_buf < 0 || s.src_buf + p.seg_copies[i] > p.n_src_bufs || s.dst_buf0 < 0 ||
                    s.dst_buf0 + p.dst_copies > p.n_dst_bufs || s.src_row0 < 0 || s.n_rows < 1 ||
                    s.src_row0 + s.n_rows > p.src_rows[s.src_buf] || s.dst_row0 < 0 ||
                    s.dst_row0 + (s.n_rows - 1) * s.dst_row_stride >= p.dst_rows_per_buf) {
                    printf("segment out of bounds at iteration %d\n", it);
                    return 1;
                }
            }
        } else ++bad;
    }
    printf("accepted %ld rejected %ld\n", ok, bad);
    return 0;
}
