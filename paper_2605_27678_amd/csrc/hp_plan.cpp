// Host-side plan builder: turns two module grids and a token map into the
// segment and tile tables the gfx950 kernels consume.  Pure C++, no HIP calls.
//
// The step it implements is the one the paper describes for communicator
// construction (Colocated communicator, second paragraph: derive every rank's
// source coordinate, destination coordinate and batch interval from G_u, G_v;
// Non-colocated communicator: both sides construct the same static routing
// pattern) plus the recorded metadata of the reverse transform ("Pipeline
// schedule details", phase 1).  Because the tables list (source run ->
// destination run) pairs, the same table drives forward and backward.
#include "hp_plan.hpp"

#include <algorithm>
#include <cstring>
#include <limits>
#include <new>
#include <numeric>

namespace hp {

Options &options() {
    static Options o;
    return o;
}

namespace {

// Position of one fused-sequence token on the destination side.
struct DstPos {
    int32_t buf0;   // first buffer that holds it
    int64_t s_loc;  // position inside that buffer's local sequence
    int64_t run;    // tokens from here on that stay consecutive in this buffer
};

// Walks the destination grid's definition for sample-local position s of a
// sample owned by dp rank `dp`.
struct DstWalker {
    int32_t tp, cp, mode, split;
    int64_t per_cp;   // positions per cp rank
    int64_t chunk;    // zigzag chunk length
    int64_t piece;    // positions per buffer (per_cp, or per_cp/tp when sharded)

    DstWalker(const hp_layout_t &g, int64_t seq)
        : tp(g.tp), cp(g.cp), mode(g.tp_mode), split(g.cp_split) {
        per_cp = seq / cp;
        chunk = (split == HP_CP_ZIGZAG) ? seq / (2 * (int64_t)cp) : per_cp;
        piece = (mode == HP_TP_SEQ_SHARD) ? per_cp / tp : per_cp;
    }

    DstPos at(int32_t dp, int64_t s) const {
        int64_t q = s / chunk, r = s - q * chunk;
        int32_t c;
        int64_t in_cp;
        if (split == HP_CP_ZIGZAG) {
            // chunks 0..C-1 are the first halves of ranks 0..C-1, chunks C..2C-1
            // are the second halves of ranks C-1..0
            if (q < cp) { c = (int32_t)q; in_cp = r; }
            else        { c = (int32_t)(2 * (int64_t)cp - 1 - q); in_cp = chunk + r; }
        } else {
            c = (int32_t)q; in_cp = r;
        }
        DstPos p;
        p.run = chunk - r;
        int32_t slice = c + cp * dp;
        if (mode == HP_TP_SEQ_SHARD) {
            int64_t t = in_cp / piece;
            p.s_loc = in_cp - t * piece;
            p.run = std::min<int64_t>(p.run, piece - p.s_loc);
            p.buf0 = (int32_t)t + tp * slice;
        } else {
            p.s_loc = in_cp;
            p.buf0 = tp * slice;
        }
        return p;
    }
};

int validate(const hp_layout_t *src, const hp_layout_t *dst, const hp_token_map_t *m) {
    if (!src || !dst || !m) return HP_EINVAL;
    for (const hp_layout_t *g : {src, dst}) {
        if (g->tp < 1 || g->cp < 1 || g->dp < 1 || g->pp < 1 || g->rank_offset < 0) return HP_EINVAL;
        if (g->tp_mode != HP_TP_REPLICATE && g->tp_mode != HP_TP_SEQ_SHARD) return HP_EINVAL;
        if (g->cp_split != HP_CP_CONTIGUOUS && g->cp_split != HP_CP_ZIGZAG) return HP_EINVAL;
        if (g->row_order != HP_ROW_BSH && g->row_order != HP_ROW_SBH) return HP_EINVAL;
    }
    if (m->batch < 1 || m->seq < 1 || m->hidden < 1 || m->n_images < 0) return HP_EINVAL;
    if (m->dtype != HP_BF16) return HP_EINVAL;
    if (m->n_images > 0 && (!m->img_sample || !m->img_start || !m->img_len)) return HP_EINVAL;

    // the encoder side has no context parallelism and plain replicated TP
    if (src->cp != 1 || src->tp_mode || src->cp_split || src->row_order) return HP_ELAYOUT;
    if (m->batch % dst->dp) return HP_ELAYOUT;
    if (m->seq % dst->cp) return HP_ELAYOUT;
    if (dst->cp_split == HP_CP_ZIGZAG && m->seq % (2 * (int64_t)dst->cp)) return HP_ELAYOUT;
    if (dst->tp_mode == HP_TP_SEQ_SHARD && (m->seq / dst->cp) % dst->tp) return HP_ELAYOUT;
    int64_t n_src = (int64_t)src->tp * src->dp;
    int64_t n_dst = (int64_t)dst->tp * dst->cp * dst->dp;
    if (n_src + n_dst > HP_MAX_BUFFERS) return HP_ELAYOUT;
    if (dst->tp_mode == HP_TP_REPLICATE && dst->tp > HP_MAX_TP) return HP_ELAYOUT;

    // spans
    int32_t prev_sample = 0, prev_dp = 0;
    for (int32_t k = 0; k < m->n_images; ++k) {
        int32_t b = m->img_sample[k];
        int64_t s = m->img_start[k], n = m->img_len[k];
        if (b < 0 || b >= m->batch || b < prev_sample) return HP_EMAP;
        if (s < 0 || n < 1 || s + n > m->seq) return HP_EMAP;
        prev_sample = b;
        if (m->img_src_dp) {
            int32_t d = m->img_src_dp[k];
            if (d < 0 || d >= src->dp || d < prev_dp) return HP_EMAP;
            prev_dp = d;
        }
    }
    // overlap inside a sample: order each sample's spans by start
    std::vector<int32_t> order(m->n_images);
    std::iota(order.begin(), order.end(), 0);
    std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        if (m->img_sample[a] != m->img_sample[b]) return m->img_sample[a] < m->img_sample[b];
        return m->img_start[a] < m->img_start[b];
    });
    for (size_t i = 1; i < order.size(); ++i) {
        int32_t a = order[i - 1], b = order[i];
        if (m->img_sample[a] == m->img_sample[b] &&
            (int64_t)m->img_start[a] + m->img_len[a] > m->img_start[b])
            return HP_EMAP;
    }
    return HP_OK;
}

void make_tiles(hp_plan *p) {
    const int64_t rb = p->row_bytes;
    int64_t tile = std::max<int64_t>(256, options().tile_bytes / 256 * 256);
    p->tiles.clear();
    for (const hp_segment_t &s : p->segments) {
        const uint64_t src0 = (uint64_t)s.src_row0 * rb, dst0 = (uint64_t)s.dst_row0 * rb;
        if (s.dst_row_stride == 1) {
            const int64_t total = s.n_rows * rb;
            for (int64_t o = 0; o < total; o += tile) {
                Tile t{};
                t.src_off = src0 + o;
                t.dst_off = dst0 + o;
                t.nbytes = (uint32_t)std::min<int64_t>(tile, total - o);
                t.pitch_rows = 1;
                t.src_buf = (uint16_t)s.src_buf;
                t.dst_buf0 = (uint16_t)s.dst_buf0;
                p->tiles.push_back(t);
            }
        } else {
            const int64_t rows_per = std::max<int64_t>(1, tile / rb);
            for (int64_t r = 0; r < s.n_rows; r += rows_per) {
                Tile t{};
                t.src_off = src0 + (uint64_t)r * rb;
                t.dst_off = dst0 + (uint64_t)r * s.dst_row_stride * rb;
                t.nbytes = (uint32_t)(std::min<int64_t>(rows_per, s.n_rows - r) * rb);
                t.pitch_rows = (uint32_t)s.dst_row_stride;
                t.src_buf = (uint16_t)s.src_buf;
                t.dst_buf0 = (uint16_t)s.dst_buf0;
                p->tiles.push_back(t);
            }
        }
    }
}

}  // namespace

int build_host_plan(const hp_layout_t *src, const hp_layout_t *dst,
                    const hp_token_map_t *m, hp_plan *p) {
    int rc = validate(src, dst, m);
    if (rc != HP_OK) return rc;

    p->src = *src;
    p->dst = *dst;
    p->batch = m->batch; p->seq = m->seq; p->hidden = m->hidden; p->dtype = m->dtype;
    p->elem_bytes = 2;
    p->row_bytes = (int64_t)m->hidden * p->elem_bytes;
    if (p->row_bytes > (int64_t)1 << 24) return HP_ELAYOUT;       // a tile holds whole rows in 32 bits
    p->n_src_bufs = src->tp * src->dp;
    p->n_dst_bufs = dst->tp * dst->cp * dst->dp;
    p->src_copies = src->tp;
    p->dst_copies = dst->tp_mode == HP_TP_SEQ_SHARD ? 1 : dst->tp;

    const DstWalker walk(*dst, m->seq);
    const int64_t b_loc = m->batch / dst->dp;                      // samples per destination dp rank
    p->dst_rows_per_buf = b_loc * walk.piece;
    const bool sbh = dst->row_order == HP_ROW_SBH;
    const int64_t stride = (sbh && b_loc > 1) ? b_loc : 1;

    // source side: each dp rank's buffer fills up in global image order
    std::vector<int64_t> fill(src->dp, 0);
    const int64_t K = m->n_images;
    int32_t d = 0;
    p->n_rows = 0;
    p->segments.clear();
    for (int64_t k = 0; k < K; ++k) {
        if (m->img_src_dp) {
            d = m->img_src_dp[k];
        } else {
            while (k >= ((int64_t)(d + 1) * K) / src->dp) ++d;    // next balanced interval
        }
        const int32_t b = m->img_sample[k];
        const int32_t dpd = (int32_t)(b / b_loc);
        const int64_t bl = b - (int64_t)dpd * b_loc;
        int64_t s = m->img_start[k], left = m->img_len[k];
        while (left > 0) {
            const DstPos pos = walk.at(dpd, s);
            const int64_t n = std::min(left, pos.run);
            hp_segment_t seg;
            seg.src_buf = d * src->tp;
            seg.dst_buf0 = pos.buf0;
            seg.src_row0 = fill[d];
            seg.dst_row0 = sbh ? pos.s_loc * b_loc + bl : bl * walk.piece + pos.s_loc;
            seg.n_rows = n;
            seg.dst_row_stride = stride;
            bool merged = false;
            if (!p->segments.empty()) {
                hp_segment_t &q = p->segments.back();
                if (q.src_buf == seg.src_buf && q.dst_buf0 == seg.dst_buf0 &&
                    q.dst_row_stride == seg.dst_row_stride &&
                    q.src_row0 + q.n_rows == seg.src_row0 &&
                    q.dst_row0 + q.n_rows * q.dst_row_stride == seg.dst_row0) {
                    q.n_rows += n;
                    merged = true;
                }
            }
            if (!merged) p->segments.push_back(seg);
            fill[d] += n;
            p->n_rows += n;
            s += n;
            left -= n;
        }
    }
    p->src_rows.assign(p->n_src_bufs, 0);
    for (int32_t dd = 0; dd < src->dp; ++dd)
        for (int32_t t = 0; t < src->tp; ++t) p->src_rows[t + src->tp * dd] = fill[dd];

    make_tiles(p);
    if (p->tiles.size() > (size_t)std::numeric_limits<int32_t>::max()) return HP_ELAYOUT;
    return HP_OK;
}

}  // namespace hp
