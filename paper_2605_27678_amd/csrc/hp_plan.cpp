// Host-side plan builder: turns two module grids and one or more token maps
// into the segment tables the gfx950 kernels consume.  Pure C++, no HIP calls.
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

std::mutex &options_mutex() {
    static std::mutex m;
    return m;
}

int tile_variant_of(int64_t tile_bytes) {
    for (int v = 0; v < kTileVariants; ++v)
        if (tile_bytes == (int64_t)tile_bytes_of(v)) return v;
    return -1;
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
    if (m->dtype != HP_BF16 && m->dtype != HP_F32) return HP_EINVAL;
    if (m->n_images > 0 && (!m->img_sample || !m->img_start || !m->img_len)) return HP_EINVAL;

    // the encoder side has no context parallelism and plain replicated TP
    if (src->cp != 1 || src->tp_mode || src->cp_split || src->row_order) return HP_ELAYOUT;
    if (m->batch % dst->dp) return HP_ELAYOUT;
    if (m->seq % dst->cp) return HP_ELAYOUT;
    if (dst->cp_split == HP_CP_ZIGZAG && m->seq % (2 * (int64_t)dst->cp)) return HP_ELAYOUT;
    if (dst->tp_mode == HP_TP_SEQ_SHARD && (m->seq / dst->cp) % dst->tp) return HP_ELAYOUT;
    if ((int64_t)src->tp * src->dp + (int64_t)dst->tp * dst->cp * dst->dp > HP_MAX_BUFFERS) return HP_ELAYOUT;
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

// Tiles of `tile` bytes needed by a segment: dense segments are cut by bytes.
// Row-strided ones are cut row by row: a row at least one tile long is cut into
// ceil(row / tile) dense pieces, shorter rows are grouped tile / row to a tile.
// The kernels use the same formulas.
uint64_t tiles_of(const hp_segment_t &s, int64_t row_bytes, uint32_t tile) {
    if (s.dst_row_stride == 1) return ((uint64_t)s.n_rows * row_bytes + tile - 1) / tile;
    if ((uint64_t)row_bytes >= tile) return (uint64_t)s.n_rows * (((uint64_t)row_bytes + tile - 1) / tile);
    const uint64_t rows_per = tile / (uint64_t)row_bytes;
    return ((uint64_t)s.n_rows + rows_per - 1) / rows_per;
}

int make_tables(hp_plan *p) {
    const size_t n = p->segments.size();
    p->dsegs.resize(n);
    for (size_t i = 0; i < n; ++i) {
        const hp_segment_t &s = p->segments[i];
        Seg &d = p->dsegs[i];
        d.src_off = (uint64_t)s.src_row0 * p->row_bytes;
        d.dst_off = (uint64_t)s.dst_row0 * p->row_bytes;
        if (s.n_rows < 1 || s.n_rows > (int64_t)kMaxSegRows || s.dst_row_stride < 1 ||
            s.dst_row_stride > (int64_t)UINT32_MAX || s.src_buf > UINT16_MAX || s.dst_buf0 > UINT16_MAX)
            return HP_ELAYOUT;                                // would not fit the descriptor's fields
        d.n_rows = (uint32_t)s.n_rows;
        d.src_copies = (uint32_t)p->seg_copies[i];
        d.pitch_rows = (uint32_t)s.dst_row_stride;
        d.src_buf = (uint16_t)s.src_buf;
        d.dst_buf0 = (uint16_t)s.dst_buf0;
    }
    p->first_tile.assign((size_t)kTileVariants * (n + 1), 0u);
    for (int v = 0; v < kTileVariants; ++v) {
        uint64_t acc = 0;
        uint32_t *row = p->first_tile.data() + (size_t)v * (n + 1);
        for (size_t i = 0; i < n; ++i) {
            row[i] = (uint32_t)acc;
            acc += tiles_of(p->segments[i], p->row_bytes, tile_bytes_of(v));
            if (acc > 0x7fffffffull) return HP_ELAYOUT;        // grid size limit
        }
        row[n] = (uint32_t)acc;
    }
    // 16-ary search trees over the keys of each variant
    p->tree.clear();
    for (int v = 0; v < kTileVariants && n > 0; ++v) {
        const uint32_t *keys = p->first_tile.data() + (size_t)v * (n + 1);
        std::vector<std::vector<uint32_t>> levels;
        levels.emplace_back(keys, keys + n);
        while (levels.back().size() > (size_t)kTreeFanout) {
            const std::vector<uint32_t> &below = levels.back();
            std::vector<uint32_t> up;
            for (size_t j = 0; j < below.size(); j += kTreeFanout) up.push_back(below[j]);
            levels.push_back(std::move(up));
        }
        if (levels.size() > (size_t)kMaxTreeLevels) return HP_ELAYOUT;
        TreeInfo &ti = p->tree_info[v];
        ti.n_levels = (uint32_t)levels.size();
        for (size_t l = 0; l < levels.size(); ++l) {
            std::vector<uint32_t> &lv = levels[l];
            lv.resize((lv.size() + kTreeFanout - 1) / kTreeFanout * kTreeFanout, 0xffffffffu);
            ti.level_off[l] = (uint32_t)p->tree.size();
            p->tree.insert(p->tree.end(), lv.begin(), lv.end());
        }
    }
    return HP_OK;
}

// Launch shapes for a new plan.  Both kernels are fastest when roughly 100 KB
// of traffic per compute unit is in flight, so the resident-wave cap that suits
// a plan falls as the number of buffers a row's traffic spreads over rises:
// 1 + dst_copies for forward, dst_copies + src_copies for backward.  The table
// is what the measured search (hp_plan_tune) picks most often per replica count
// on the five workloads and their sequence-sharded variants; an option that is
// not HP_AUTO overrides its field.
void default_launches(hp_plan *p) {
    Options o;
    {
        std::lock_guard<std::mutex> lk(options_mutex());
        o = options();
    }
    const int c = p->dst_copies, s = p->src_copies;
    Launch f{1, 64, c <= 1 ? 24 : c <= 4 ? 12 : c <= 7 ? 8 : 5, 2};                          // 2 KiB tiles
    if (c == 2) f = Launch{2, 256, 28, 2};      // two copies: 4 KiB tiles, 256 lanes (+3.6 % on config 4 over 2 KiB x 64, cap 14)
    Launch b = c + s <= 2 ? Launch{1, 64, 30, 3} : c + s == 3 ? Launch{0, 64, 30, 3} : Launch{0, 64, 16, 3};
    // accumulating backward: the binary32 accumulators are read and written, 2 * 4 / elem_bytes row sizes per copy;
    // caps as the measured search finds them for 6, 8 and 16 streams (configs 4, 3 and 5)
    const int acc_streams = c + s * 8 / p->elem_bytes;
    Launch a{1, 64, acc_streams <= 4 ? 16 : acc_streams <= 6 ? 13 : acc_streams <= 8 ? 11 : acc_streams <= 12 ? 9 : 7, 3};
    auto apply = [](Launch &L, int64_t tile, int64_t block, int64_t waves, int64_t nt) {
        if (tile > 0) L.tile_variant = tile_variant_of(tile);
        if (block > 0) L.block = (int32_t)block;
        if (waves >= 0) L.waves_per_cu = (int32_t)waves;
        L.nontemporal = (int32_t)nt;
    };
    apply(f, o.tile_bytes_fwd, o.block_threads_fwd, o.waves_per_cu_fwd, o.nontemporal_fwd);
    apply(b, o.tile_bytes_bwd, o.block_threads_bwd, o.waves_per_cu_bwd, o.nontemporal_bwd);
    apply(a, o.tile_bytes_bwd > 0 ? std::max<int64_t>(o.tile_bytes_bwd, 4096) : -1, o.block_threads_bwd,
          o.waves_per_cu_bwd, o.nontemporal_bwd);
    p->fwd = f;
    p->bwd = b;
    p->acc = a;
}

// No two spans of one microbatch may overlap, whichever edge they belong to.
int check_cross_edge_overlap(const hp_token_map_t *maps, int32_t n_edges, int32_t n_maps) {
    struct Span { int32_t b; int64_t s, e; };
    std::vector<Span> spans;
    for (int32_t mi = 0; mi < n_maps; ++mi) {
        spans.clear();
        for (int32_t e = 0; e < n_edges; ++e) {
            const hp_token_map_t &m = maps[(size_t)e * n_maps + mi];
            for (int32_t k = 0; k < m.n_images; ++k)
                spans.push_back(Span{m.img_sample[k], m.img_start[k], (int64_t)m.img_start[k] + m.img_len[k]});
        }
        std::sort(spans.begin(), spans.end(), [](const Span &x, const Span &y) {
            return x.b != y.b ? x.b < y.b : x.s < y.s;
        });
        for (size_t i = 1; i < spans.size(); ++i)
            if (spans[i].b == spans[i - 1].b && spans[i].s < spans[i - 1].e) return HP_EMAP;
    }
    return HP_OK;
}

}  // namespace

int build_host_plan(const hp_layout_t *srcs, int32_t n_edges, const hp_layout_t *dst,
                    const hp_token_map_t *maps, int32_t n_maps, hp_plan *p) {
    if (!srcs || !maps || n_maps < 1 || n_edges < 1) return HP_EINVAL;
    int64_t n_bufs = 0;
    for (int32_t e = 0; e < n_edges; ++e) {
        for (int32_t i = 0; i < n_maps; ++i) {
            const hp_token_map_t &m = maps[(size_t)e * n_maps + i];
            int rc = validate(&srcs[e], dst, &m);
            if (rc != HP_OK) return rc;
            // microbatches and edges share the buffer shapes
            if (m.batch != maps[0].batch || m.seq != maps[0].seq || m.hidden != maps[0].hidden ||
                m.dtype != maps[0].dtype)
                return HP_ELAYOUT;
        }
        n_bufs += (int64_t)srcs[e].tp * srcs[e].dp * n_maps;
    }
    n_bufs += (int64_t)dst->tp * dst->cp * dst->dp * n_maps;
    if (n_bufs > HP_MAX_BUFFERS) return HP_ELAYOUT;
    if (n_edges > 1) {
        int rc = check_cross_edge_overlap(maps, n_edges, n_maps);
        if (rc != HP_OK) return rc;
    }
    const hp_token_map_t *m0 = &maps[0];

    p->src = srcs[0];
    p->dst = *dst;
    p->batch = m0->batch; p->seq = m0->seq; p->hidden = m0->hidden; p->dtype = m0->dtype;
    p->n_maps = n_maps;
    p->n_edges = n_edges;
    p->elem_bytes = m0->dtype == HP_F32 ? 4 : 2;
    p->row_bytes = (int64_t)m0->hidden * p->elem_bytes;
    if (p->row_bytes > (int64_t)1 << 24) return HP_ELAYOUT;       // a tile holds whole rows in 32 bits
    const int32_t dst_per_map = dst->tp * dst->cp * dst->dp;
    p->n_dst_bufs = dst_per_map * n_maps;
    p->src_copies = srcs[0].tp;
    p->dst_copies = dst->tp_mode == HP_TP_SEQ_SHARD ? 1 : dst->tp;

    const DstWalker walk(*dst, m0->seq);
    const int64_t b_loc = m0->batch / dst->dp;                     // samples per destination dp rank
    p->dst_rows_per_buf = b_loc * walk.piece;
    const bool sbh = dst->row_order == HP_ROW_SBH;
    const int64_t stride = (sbh && b_loc > 1) ? b_loc : 1;

    p->n_rows = 0;
    p->bwd_bytes = p->bwd_accum_bytes = 0;
    p->segments.clear();
    p->seg_copies.clear();
    p->src_rows.clear();
    p->src_leader.clear();
    int32_t edge_base = 0;
    for (int32_t e = 0; e < n_edges; ++e) {
        const hp_layout_t *src = &srcs[e];
        const int32_t src_per_map = src->tp * src->dp;
        p->src_rows.resize((size_t)edge_base + (size_t)src_per_map * n_maps, 0);
        p->src_leader.resize(p->src_rows.size(), 0);
        int64_t edge_rows = 0;
        for (int32_t mi = 0; mi < n_maps; ++mi) {
            const hp_token_map_t *m = &maps[(size_t)e * n_maps + mi];
            const int32_t src_base = edge_base + mi * src_per_map, dst_base = mi * dst_per_map;
            // source side: each dp rank's buffer fills up in global image order
            std::vector<int64_t> fill(src->dp, 0);
            const int64_t K = m->n_images;
            int32_t d = 0;
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
                    seg.src_buf = src_base + d * src->tp;
                    seg.dst_buf0 = dst_base + pos.buf0;
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
                            q.dst_row0 + q.n_rows * q.dst_row_stride == seg.dst_row0 &&
                            q.n_rows + n <= (int64_t)kMaxSegRows) {   // the device descriptor counts rows in 32 bits
                            q.n_rows += n;
                            merged = true;
                        }
                    }
                    if (!merged) {
                        p->segments.push_back(seg);
                        p->seg_copies.push_back(src->tp);
                    }
                    fill[d] += n;
                    edge_rows += n;
                    s += n;
                    left -= n;
                }
            }
            for (int32_t dd = 0; dd < src->dp; ++dd)
                for (int32_t t = 0; t < src->tp; ++t) {
                    p->src_rows[src_base + t + src->tp * dd] = fill[dd];
                    p->src_leader[src_base + t + src->tp * dd] = t == 0;
                }
        }
        p->n_rows += edge_rows;
        const int64_t edge_bytes = edge_rows * p->row_bytes;
        p->bwd_bytes += ((int64_t)p->dst_copies + src->tp) * edge_bytes;
        p->bwd_accum_bytes += (int64_t)p->dst_copies * edge_bytes + (int64_t)src->tp * 2 * edge_rows * p->hidden * 4;
        edge_base += src_per_map * n_maps;
    }
    p->n_src_bufs = edge_base;

    default_launches(p);
    return make_tables(p);
}

}  // namespace hp
