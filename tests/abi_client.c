/* A plain C99 client of the library's C ABI (no HIP header, no C++): builds a
 * host-only plan for the long-context grids, reads it back through the query
 * calls and checks the error paths.  Compiled with gcc and linked against
 * libhp.so by tests/test_cli_and_loading.py; makes no GPU call. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "hp.h"

#define CHECK(c) do { if (!(c)) { printf("line %d: %s\n", __LINE__, #c); return 1; } } while (0)

int main(void)
{
    hp_layout_t src, dst;
    hp_token_map_t map;
    hp_plan_t *plan = NULL;
    hp_plan_info_t info;
    int32_t sample[3] = {0, 0, 0}, start[3] = {100, 9000, 70000}, len[3] = {576, 2304, 1024};
    int64_t rows[8];
    hp_segment_t segs[16];
    hp_launch_t shape;
    int n, i;
    int64_t total = 0;

    memset(&src, 0, sizeof src); memset(&dst, 0, sizeof dst); memset(&map, 0, sizeof map);
    src.tp = 1; src.cp = 1; src.dp = 8; src.pp = 1;
    dst.tp = 4; dst.cp = 8; dst.dp = 1; dst.pp = 1; dst.cp_split = HP_CP_ZIGZAG;
    map.batch = 1; map.seq = 131072; map.hidden = 5120; map.dtype = HP_BF16;
    map.n_images = 3; map.img_sample = sample; map.img_start = start; map.img_len = len;

    CHECK(hp_plan_create_host(&src, &dst, &map, &plan) == HP_OK && plan != NULL);
    CHECK(hp_plan_query(plan, &info) == HP_OK);
    CHECK(info.n_src_bufs == 8 && info.n_dst_bufs == 32 && info.dst_copies == 4 && info.src_copies == 1);
    CHECK(info.n_rows == 576 + 2304 + 1024 && info.row_bytes == 10240 && info.dst_rows_per_buf == 16384);
    CHECK(info.fwd_bytes == 5 * info.boundary_bytes && info.bwd_bytes == 5 * info.boundary_bytes);
    CHECK(info.on_device == 0 && info.device == -1);
    CHECK(hp_plan_src_rows(plan, rows, 8) == 8);
    for (i = 0; i < 8; ++i) total += rows[i];
    CHECK(total == info.n_rows);
    n = hp_plan_segments(plan, segs, 16);
    CHECK(n == info.n_segments && n >= 3 && n <= 16);
    total = 0;
    for (i = 0; i < n; ++i) {
        CHECK(segs[i].n_rows > 0 && segs[i].dst_row_stride == 1);
        CHECK(segs[i].dst_buf0 % 4 == 0 && segs[i].dst_buf0 < 32 && segs[i].src_buf < 8);
        CHECK(segs[i].dst_row0 + segs[i].n_rows <= info.dst_rows_per_buf);
        total += segs[i].n_rows;
    }
    CHECK(total == info.n_rows);
    CHECK(hp_plan_get_launch(plan, 0, &shape) == HP_OK && shape.tile_bytes == 2048 && shape.block_threads == 64);
    shape.tile_bytes = 3000;
    CHECK(hp_plan_set_launch(plan, 0, &shape) == HP_EINVAL);
    {   /* a host-only plan cannot be launched; nothing is written through the null tables */
        const void *s8[8] = {0}; void *d32[32] = {0};
        CHECK(hp_forward(plan, s8, d32, NULL) == HP_EINVAL || hp_forward(plan, s8, d32, NULL) == HP_ESTATE);
    }
    hp_plan_destroy(plan);
    plan = NULL;
    map.seq = 131071;                                   /* does not divide over 2 x 8 zigzag chunks */
    CHECK(hp_plan_create_host(&src, &dst, &map, &plan) == HP_ELAYOUT && plan == NULL);
    map.seq = 131072; len[2] = 70000;                   /* span runs past the end of the sequence */
    CHECK(hp_plan_create_host(&src, &dst, &map, &plan) == HP_EMAP && plan == NULL);
    CHECK(strstr(hp_strerror(HP_EMAP), "token map") != NULL && strstr(hp_version(), "gfx950") != NULL);
    hp_plan_destroy(NULL);
    printf("abi client ok: %d segments\n", n);
    return 0;
}
