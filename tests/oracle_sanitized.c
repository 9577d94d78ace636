/* Driver that runs the CPU oracle (oracle/hp_oracle.c, compiled into this
 * program with ASan + UBSan by tests/test_oracle_sanitized.py) on cases read
 * from a file, with every buffer allocated at its exact size so that any
 * out-of-bounds access of the oracle is reported.  Results go to a second file
 * and are compared in Python with the fixtures and with the ordinary build.
 *
 * input:  int32 n_cases, then per case
 *           int32 src[6], dst[6]          (tp, cp, dp, tp_mode, cp_split, row_order)
 *           int32 batch, seq, hidden, n_images, has_src_dp
 *           int32 img_sample[n], img_start[n], img_len[n] (, img_src_dp[n])
 *           uint16 source buffers, destination prefill, destination gradients
 *           (each buffer in index order, rows as the oracle reports them)
 * output: per case uint16 destination buffers after forward, uint16 source
 *         gradients (orc_backward_bf16), uint16 source gradients (orc_backward,
 *         bf16 overwrite), float accumulators after orc_backward(accumulate) from
 *         zero, int32/int64 forward map of destination buffer 0.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct { int32_t tp, cp, dp, tp_mode, cp_split, row_order; } orc_grid_t;
typedef struct {
    int32_t batch, seq, hidden, n_images;
    const int32_t *img_sample, *img_start, *img_len, *img_src_dp;
} orc_map_t;

int64_t orc_src_rows(const orc_grid_t *, const orc_map_t *, int32_t);
int64_t orc_dst_rows(const orc_grid_t *, const orc_map_t *);
int orc_forward_map(const orc_grid_t *, const orc_grid_t *, const orc_map_t *, int32_t, int32_t *, int64_t *);
int orc_forward(const orc_grid_t *, const orc_grid_t *, const orc_map_t *, int32_t, const void *const *, void *const *);
int orc_backward(const orc_grid_t *, const orc_grid_t *, const orc_map_t *, int32_t, int32_t,
                 const void *const *, void *const *);
int orc_backward_bf16(const orc_grid_t *, const orc_grid_t *, const orc_map_t *, const uint16_t *const *,
                      uint16_t *const *);

static void must_read(void *p, size_t n, FILE *f) { if (n && fread(p, 1, n, f) != n) { fprintf(stderr, "short input\n"); exit(3); } }
static void *exact(size_t n) { void *p = malloc(n ? n : 1); if (!p) exit(4); return p; }

int main(int argc, char **argv)
{
    if (argc < 3) return 2;
    FILE *in = fopen(argv[1], "rb"), *out = fopen(argv[2], "wb");
    if (!in || !out) return 2;
    int32_t n_cases;
    must_read(&n_cases, 4, in);
    for (int32_t c = 0; c < n_cases; ++c) {
        orc_grid_t src, dst;
        int32_t hdr[5];
        must_read(&src, sizeof src, in);
        must_read(&dst, sizeof dst, in);
        must_read(hdr, sizeof hdr, in);
        const int32_t n = hdr[3];
        int32_t *smp = exact(4 * (size_t)n), *st = exact(4 * (size_t)n), *ln = exact(4 * (size_t)n), *dp = NULL;
        must_read(smp, 4 * (size_t)n, in); must_read(st, 4 * (size_t)n, in); must_read(ln, 4 * (size_t)n, in);
        if (hdr[4]) { dp = exact(4 * (size_t)n); must_read(dp, 4 * (size_t)n, in); }
        orc_map_t m = { hdr[0], hdr[1], hdr[2], n, smp, st, ln, dp };
        const size_t H = (size_t)m.hidden;
        const int n_src = src.tp * src.dp, n_dst = dst.tp * dst.cp * dst.dp;
        const size_t drows = (size_t)orc_dst_rows(&dst, &m);
        void **sb = exact(sizeof(void *) * n_src), **db = exact(sizeof(void *) * n_dst), **gb = exact(sizeof(void *) * n_dst);
        void **sg = exact(sizeof(void *) * n_src), **sg2 = exact(sizeof(void *) * n_src), **acc = exact(sizeof(void *) * n_src);
        size_t *srows = exact(sizeof(size_t) * n_src);
        for (int i = 0; i < n_src; ++i) {
            srows[i] = (size_t)orc_src_rows(&src, &m, i / src.tp);
            sb[i] = exact(2 * srows[i] * H);
            must_read(sb[i], 2 * srows[i] * H, in);
            sg[i] = exact(2 * srows[i] * H);  memset(sg[i], 0xEE, 2 * srows[i] * H);
            sg2[i] = exact(2 * srows[i] * H); memset(sg2[i], 0xEE, 2 * srows[i] * H);
            acc[i] = exact(4 * srows[i] * H); memset(acc[i], 0, 4 * srows[i] * H);
        }
        for (int j = 0; j < n_dst; ++j) { db[j] = exact(2 * drows * H); must_read(db[j], 2 * drows * H, in); }
        for (int j = 0; j < n_dst; ++j) { gb[j] = exact(2 * drows * H); must_read(gb[j], 2 * drows * H, in); }
        int32_t *fm_buf = exact(4 * drows); int64_t *fm_row = exact(8 * drows);
        int rc = orc_forward(&src, &dst, &m, 2, (const void *const *)sb, db);
        rc |= orc_backward_bf16(&src, &dst, &m, (const uint16_t *const *)gb, (uint16_t *const *)sg);
        rc |= orc_backward(&src, &dst, &m, 0, 0, (const void *const *)gb, sg2);
        rc |= orc_backward(&src, &dst, &m, 0, 1, (const void *const *)gb, acc);
        rc |= orc_forward_map(&src, &dst, &m, 0, fm_buf, fm_row);
        if (rc) { fprintf(stderr, "case %d: oracle refused the layout\n", c); return 5; }
        for (int j = 0; j < n_dst; ++j) fwrite(db[j], 2, drows * H, out);
        for (int i = 0; i < n_src; ++i) fwrite(sg[i], 2, srows[i] * H, out);
        for (int i = 0; i < n_src; ++i) fwrite(sg2[i], 2, srows[i] * H, out);
        for (int i = 0; i < n_src; ++i) fwrite(acc[i], 4, srows[i] * H, out);
        fwrite(fm_buf, 4, drows, out); fwrite(fm_row, 8, drows, out);
        for (int i = 0; i < n_src; ++i) { free(sb[i]); free(sg[i]); free(sg2[i]); free(acc[i]); }
        for (int j = 0; j < n_dst; ++j) { free(db[j]); free(gb[j]); }
        free(sb); free(db); free(gb); free(sg); free(sg2); free(acc); free(srows); free(fm_buf); free(fm_row);
        free(smp); free(st); free(ln); free(dp);
    }
    fclose(in);
    if (fclose(out)) return 6;
    printf("cases %d\n", n_cases);
    return 0;
}
