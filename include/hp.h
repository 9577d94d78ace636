/*
 * hp.h - C ABI of the heterogeneous-parallelism boundary layout transform for
 * AMD MI355X (gfx950).
 *
 * The operation (paper, Method section, paragraph on boundary edges): an edge
 * u -> v between two modules carries ONE tensor with TWO distributed
 * representations, one under the source module's grid G_u on ranks R_u and one
 * under the destination module's grid G_v on ranks R_v.  Forward materialises
 * the activation in the destination layout; backward applies the matching
 * reverse transform so that gradients return to the source layout.  Here u is a
 * vision encoder (TP x DP grid, CP = 1) and v is the language model
 * (TP x CP x DP grid): the encoder's projected tokens are inserted into the
 * fused multimodal sequence at the image-token positions (Fig. 1 caption;
 * appendix "Pipeline schedule details", phase 2), the fused sequence is split
 * over the CP ranks (Introduction: CP shards the fused language sequence) and
 * the result is present on every TP rank of the receiving group
 * (Non-colocated communicator: local TP/CP broadcast to non-leader ranks).
 *
 * Every rank is emulated as its own buffer in one GPU's HBM.  The library moves
 * rows between those buffers with hand-written gfx950 kernels; it performs no
 * inter-GPU communication.
 *
 * Conventions (the paper leaves them open; they are fixed here):
 *   - Rank order inside a grid: tp fastest, then cp, then dp.  Buffer index of a
 *     source rank: tp + TP_src*dp.  Buffer index of a destination rank:
 *     tp + TP_dst*(cp + CP_dst*dp).  rank_offset only names the physical ranks
 *     (overlapping ranges = colocated, disjoint = non-colocated; appendix
 *     "Open-source user configuration example"); it does not change the result.
 *   - A source buffer is [rows, hidden]: the tokens of the images assigned to
 *     that dp rank, concatenated in global image order.  All TP ranks of one
 *     source dp rank hold identical copies; forward reads copy tp = 0 (the
 *     boundary leader), backward writes every copy.
 *   - Image -> source dp rank: the map's img_src_dp if given, else contiguous
 *     balanced intervals of the K images: rank d holds images
 *     [floor(d*K/DP), floor((d+1)*K/DP)).  With a constant number of images per
 *     sample this is the paper's equal batch intervals (Method: logical
 *     batch-shard transform).  Fan-in, fan-out and equal-DP all follow from it.
 *   - Sample b lives on destination dp rank b / (batch/DP_dst).
 *   - A destination buffer is [B_local, S_local, hidden] (HP_ROW_BSH) or
 *     [S_local, B_local, hidden] (HP_ROW_SBH), densely packed.
 *   - Backward SUMS the TP replicas of a row (the adjoint of replication):
 *     binary32 left fold in ascending tp order, round-to-nearest-even,
 *     subnormals kept, then one rounding to bf16.  (The paper's own stack
 *     returns the leader's copy without a reduction.)
 *
 * Threading / ownership: apart from its launch shapes (hp_plan_set_launch,
 * hp_plan_tune) a plan is immutable after creation and may be used from several
 * host threads and streams at once.  The caller owns every activation and
 * gradient buffer and the stream; the plan owns only its device tables (a few
 * KB).  hp_forward / hp_backward / hp_backward_accumulate enqueue one kernel on
 * the caller's stream and return without synchronising; they allocate nothing
 * and use no scratch memory.  Buffers must stay valid until the stream has
 * passed the call.  The library performs no bounds checks on the caller's
 * buffers: each must hold at least the rows hp_plan_src_rows /
 * hp_plan_query report.
 *
 * Errors: every int-returning call returns HP_OK (0) or a negative HP_E* code;
 * nothing throws or aborts across this boundary and output arguments are left
 * untouched on failure.
 */
#ifndef HP_H_
#define HP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HP_OK        0
#define HP_EINVAL   (-1)  /* null pointer, non-positive size, unknown enum value            */
#define HP_ELAYOUT  (-2)  /* grids and token map do not divide / exceed a stated limit      */
#define HP_EMAP     (-3)  /* bad image spans: out of range, overlapping, unordered samples  */
#define HP_ENOMEM   (-4)  /* host or device allocation failed                               */
#define HP_EHIP     (-5)  /* a HIP runtime call failed (see hp_last_hip_error)              */
#define HP_ESTATE   (-6)  /* plan has no device tables (host-only plan) or wrong device     */
#define HP_EALIGN   (-7)  /* a buffer pointer is not aligned to the element size            */

/* hp_layout_t.tp_mode (destination only) */
#define HP_TP_REPLICATE  0   /* every TP rank holds the full CP-local sequence               */
#define HP_TP_SEQ_SHARD  1   /* sequence parallelism: TP rank t holds the t-th of TP equal
                                contiguous pieces of the CP-local sequence; no replication  */
/* hp_layout_t.cp_split (destination only) */
#define HP_CP_CONTIGUOUS 0   /* cp rank r holds positions [r*S/C, (r+1)*S/C)                 */
#define HP_CP_ZIGZAG     1   /* load-balanced: 2C equal chunks, rank r holds chunk r followed
                                by chunk 2C-1-r                                              */
/* hp_layout_t.row_order (destination only) */
#define HP_ROW_BSH 0
#define HP_ROW_SBH 1
/* hp_token_map_t.dtype: element type of the activations and gradients */
#define HP_BF16 0
#define HP_F32  1   /* the paper validates in FP32 as well as BF16; forward moves
                       4-byte elements, backward folds them with no final rounding */

#define HP_MAX_BUFFERS 448   /* source + destination buffers of one plan, all microbatches   */
#define HP_MAX_TP      16    /* replicas summed by hp_backward                               */

/* One module's logical grid G_m and the first id of its physical rank range R_m
 * (Method, first paragraph; appendix "Open-source user configuration example").
 * pp is accepted for completeness and must be >= 1: only the boundary stage
 * (source's last stage, destination's first stage) takes part.  For the source
 * grid cp must be 1 and tp_mode/cp_split/row_order must be 0. */
typedef struct hp_layout {
    int32_t tp, cp, dp, pp;
    int32_t rank_offset;
    int32_t tp_mode;
    int32_t cp_split;
    int32_t row_order;
} hp_layout_t;

/* Shape of the fused sequence and where the image tokens sit in it.  All
 * pointers are HOST arrays of n_images entries, read during plan creation only.
 * Images are listed in global order: img_sample non-decreasing; within a sample
 * any non-overlapping placement.  Image k occupies positions
 * [img_start[k], img_start[k]+img_len[k]) of sample img_sample[k].
 * img_src_dp may be NULL (balanced rule above) or a non-decreasing array of
 * source dp ranks. */
typedef struct hp_token_map {
    int32_t batch, seq, hidden;
    int32_t dtype;                 /* HP_BF16 or HP_F32 */
    int32_t n_images;
    const int32_t *img_sample;
    const int32_t *img_start;
    const int32_t *img_len;
    const int32_t *img_src_dp;
} hp_token_map_t;

typedef struct hp_plan hp_plan_t;

typedef struct hp_plan_info {
    int32_t n_src_bufs;        /* TP_src * DP_src (times microbatches, summed over joined edges) */
    int32_t n_dst_bufs;        /* TP_dst * CP_dst * DP_dst                                    */
    int32_t src_copies;        /* TP_src: identical copies of every source row (first edge)   */
    int32_t dst_copies;        /* TP_dst when replicated, 1 when sequence-sharded             */
    int64_t n_rows;            /* N: image-token rows of the boundary tensor                  */
    int64_t row_bytes;         /* hidden * element size                                       */
    int64_t dst_rows_per_buf;  /* rows of every destination buffer                            */
    int64_t boundary_bytes;    /* N * row_bytes                                               */
    int64_t fwd_bytes;         /* algorithmic traffic of hp_forward: (1 + dst_copies)*boundary */
    int64_t bwd_bytes;         /* of hp_backward: (dst_copies + src_copies)*boundary, per edge */
    int32_t n_segments;        /* runs contiguous on both sides                               */
    int32_t n_tiles;           /* workgroups of an hp_forward launch in its current shape     */
    int32_t on_device;         /* 1 if device tables exist                                    */
    int32_t device;            /* HIP device ordinal of the tables, -1 if none                */
    int32_t n_maps;            /* microbatches folded into the plan (1 unless batched)        */
    int32_t elem_bytes;        /* 2 for HP_BF16, 4 for HP_F32                                 */
    int64_t bwd_accum_bytes;   /* algorithmic traffic of hp_backward_accumulate: dst_copies *
                                  boundary read + src_copies * N * hidden * 4 read and written */
    int32_t n_edges;           /* source modules joined into the destination (1 unless joined) */
    int32_t reserved;
} hp_plan_info_t;

/* A maximal run of image-token rows that is contiguous in the source buffer and
 * evenly strided in the destination buffer(s). */
typedef struct hp_segment {
    int32_t src_buf;           /* source buffer index of copy tp = 0                          */
    int32_t dst_buf0;          /* first destination buffer; copies are dst_buf0 .. +dst_copies-1 */
    int64_t src_row0;
    int64_t dst_row0;
    int64_t n_rows;
    int64_t dst_row_stride;    /* 1 for HP_ROW_BSH, B_local for HP_ROW_SBH                    */
} hp_segment_t;

/* hp_plan_create - the construction step of a communicator: from the two grids
 * alone every rank's place on the source side, its place on the destination
 * side and the batch interval it exchanges are worked out once and kept
 * (Colocated communicator, second paragraph; the non-colocated communicator
 * builds the same fixed routing on both sides): validates the two grids and the token map,
 * builds the segment table (runs of rows contiguous on both sides) and the
 * search trees that map a workgroup to its segment on the host, and uploads
 * them to the CURRENT HIP device (a few KB; one synchronous copy into a device
 * block that is recycled from earlier plans when one is free).
 * src, dst, map: host structs, read only during the call.
 * *out receives an owned plan; release it with hp_plan_destroy. */
int hp_plan_create(const hp_layout_t *src, const hp_layout_t *dst,
                   const hp_token_map_t *map, hp_plan_t **out);

/* Same, but makes no HIP call: the plan can be queried and its segments read,
 * hp_forward / hp_backward on it return HP_ESTATE. */
int hp_plan_create_host(const hp_layout_t *src, const hp_layout_t *dst,
                        const hp_token_map_t *map, hp_plan_t **out);

/* One plan for n_maps microbatches that share the two grids and the buffer
 * shapes (same batch, seq, hidden) but have their own token maps and their own
 * buffers - the packed boundary tensor with per-microbatch views of the
 * colocated schedule (appendix "Pipeline schedule details", phases 1-3), and
 * the per-microbatch invocations of the non-colocated communicator folded into
 * one launch per direction.  Buffer arrays are microbatch-major: source buffer
 * index m*(TP_src*DP_src) + tp + TP_src*dp, destination buffer index
 * m*(TP_dst*CP_dst*DP_dst) + tp + TP_dst*(cp + CP_dst*dp); the totals must not
 * exceed HP_MAX_BUFFERS.  host_only != 0 skips the device upload. */
int hp_plan_create_batched(const hp_layout_t *src, const hp_layout_t *dst,
                           const hp_token_map_t *maps, int32_t n_maps,
                           int32_t host_only, hp_plan_t **out);

/* One plan for a graph join: n_edges source modules (several encoders), each
 * with its own grid srcs[e], feed the same destination module, and every edge
 * is a boundary transform of its own into the one fused sequence ("Pipeline
 * schedule details": the first LLM stage consumes several encoder activations
 * for the same microbatch, and backward routes each gradient through the
 * communicator of the edge it came in by).  maps[e * n_maps + m] is edge e's
 * token map for microbatch m: where THAT encoder's tokens sit in the sequence.
 * All maps share batch, seq, hidden and dtype; spans of different edges must
 * not overlap (HP_EMAP).  One hp_forward launch scatters the tokens of every
 * edge; one hp_backward launch returns each row's gradient to its own edge's
 * source ranks, to all TP copies of that edge's grid.
 * Source buffers are listed edge by edge: edge e starts at
 * sum over e' < e of n_maps * TP_e' * DP_e', and inside the edge the index is
 * m * (TP_e * DP_e) + tp + TP_e * dp.  Destination buffers as for
 * hp_plan_create_batched, shared by all edges.  With n_edges = 1 this is
 * hp_plan_create_batched. */
int hp_plan_create_joined(const hp_layout_t *srcs, int32_t n_edges, const hp_layout_t *dst,
                          const hp_token_map_t *maps, int32_t n_maps,
                          int32_t host_only, hp_plan_t **out);

/* Frees the host tables and hands the device block (a few KB) back to a small
 * per-process cache from which later hp_plan_create calls on the same device
 * are served, so that plans can be rebuilt at training-step rate without a
 * hipMalloc / hipFree pair each time.  NULL is allowed.  The call may follow the
 * last hp_forward / hp_backward that uses the plan at once, without any
 * synchronisation: the block is not overwritten before the streams those calls
 * were enqueued on have passed them (an event per stream is recorded here and
 * waited for when the block is next handed out).  Call it with the plan's
 * device current.  Every stream the plan was used on must still exist when this
 * is called (destroy the plan before the stream, not after: the handle is
 * queried and an event is recorded on it here).  A plan whose calls were
 * recorded into a HIP graph has to outlive the replays of that graph. */
void hp_plan_destroy(hp_plan_t *plan);

/* hipFree()s every cached device block (at most 64 blocks of a few KB). */
void hp_release_cached_memory(void);

int hp_plan_query(const hp_plan_t *plan, hp_plan_info_t *info);

/* rows[i] = rows of source buffer i (i = tp + TP_src*dp).  `cap` = entries
 * available in `rows` (host array); returns the number of source buffers, or a
 * negative error.  Empty source ranks have 0 rows. */
int hp_plan_src_rows(const hp_plan_t *plan, int64_t *rows, int32_t cap);

/* Copies up to `cap` segments into `out` (host array); returns the total
 * number of segments. */
int hp_plan_segments(const hp_plan_t *plan, hp_segment_t *out, int32_t cap);

/* hp_forward - produce the source module's activation in the layout of the
 * destination module (Method, paragraph on boundary edges: the forward direction
 * of an edge; fan-in concatenation in batch order, Non-colocated communicator;
 * insertion into the text embeddings, appendix "Pipeline schedule details",
 * phase 2).
 *   src_bufs: HOST array of n_src_bufs DEVICE pointers, index tp + TP_src*dp,
 *             each [rows_i, hidden] of the plan's dtype.  Only copies with tp == 0 are read;
 *             entries of other copies and of empty ranks may be NULL.
 *   dst_bufs: HOST array of n_dst_bufs DEVICE pointers, index
 *             tp + TP_dst*(cp + CP_dst*dp), each [dst_rows_per_buf, hidden].
 *             Exactly the image-token rows are written; all other bytes (the
 *             text embeddings the caller placed there) are left as found.
 *   stream:   a hipStream_t (NULL = the default stream).  The call is ordered
 *             against work on THIS stream only: whatever produced src_bufs (and
 *             the text rows of dst_bufs) on another stream must have finished,
 *             or the caller makes `stream` wait for it first.  The same holds
 *             for every call below that takes a stream.
 * Pointers must be aligned to the element size; 16-byte alignment (with a row
 * size that is a multiple of 16) selects the vector path.  Returns after
 * enqueueing. */
int hp_forward(const hp_plan_t *plan, const void *const *src_bufs,
               void *const *dst_bufs, void *stream);

/* hp_backward - route destination-layout gradients back to the source layout
 * (Method, paragraph on boundary edges: the backward direction of an edge undoes
 * the forward layout change; fan-in backward splits along the recorded
 * intervals; the result is placed on every TP rank of the source side,
 * Non-colocated communicator, backward paragraph).
 * The dst_copies replicas of each image-token row are summed in binary32 in
 * ascending tp order and rounded once to bf16 (HP_F32: no final rounding).
 *   dst_grad_bufs: HOST array of n_dst_bufs DEVICE pointers, same shapes as
 *                  hp_forward's dst_bufs; only image-token rows are read.
 *   src_grad_bufs: HOST array of n_src_bufs DEVICE pointers; every row of
 *                  every buffer is overwritten (all TP copies get the same
 *                  values).  Entries of empty ranks may be NULL.
 */
int hp_backward(const hp_plan_t *plan, const void *const *dst_grad_bufs,
                void *const *src_grad_bufs, void *stream);

/* hp_zero_image_rows - sets exactly the image-token rows of every destination-
 * shaped buffer to zero (all dst_copies copies; every other byte is left as
 * found).  The rows that hp_forward inserts do not depend on the text
 * embeddings that were there before (appendix "Pipeline schedule details",
 * phase 2: the boundary view is put into the microbatch's text embeddings at the
 * image positions), so the gradient of the fused sequence with respect to those
 * text embeddings is the destination gradient with these rows blanked: an
 * autograd wrapper around hp_forward / hp_backward calls this on a copy of the
 * destination gradients after hp_backward has read them.
 *   dst_bufs: HOST array of n_dst_bufs DEVICE pointers, shapes as for hp_forward.
 * Uses hp_forward's launch shape; allocates nothing; returns after enqueueing. */
int hp_zero_image_rows(const hp_plan_t *plan, void *const *dst_bufs, void *stream);

/* hp_backward_accumulate - as hp_backward, but the source side holds binary32
 * gradient ACCUMULATORS that are added to instead of overwritten: the gradients
 * that accumulate on the packed boundary tensor over the microbatches of a
 * pipeline window before the encoder backward consumes them (appendix "Pipeline
 * schedule details", phase 3).  For every image-token row the replicas are
 * folded as in hp_backward (ascending tp, binary32, no rounding to the gradient
 * dtype) and the sum s is applied as acc = acc + s to every source TP copy.
 *   dst_grad_bufs:  as for hp_backward (bf16 or f32 per the plan's dtype).
 *   src_accum_bufs: HOST array of n_src_bufs DEVICE pointers to binary32 arrays
 *                   [rows_i, hidden], read and written; 4-byte aligned (16-byte
 *                   alignment and hidden % 4 == 0 select the vector path).
 * Has its own launch shape (direction 2). */
int hp_backward_accumulate(const hp_plan_t *plan, const void *const *dst_grad_bufs,
                           void *const *src_accum_bufs, void *stream);

/* hp_forward_static - hp_forward for callers that cannot allocate device memory
 * or let the library do so: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  hp_forward reads its plan's tables from a
 * device block that hp_plan_create allocated; this call instead takes ANY plan
 * (normally a host-only one from hp_plan_create_host or the host_only variants,
 * whose creation makes no HIP call), writes the tables this launch needs - the
 * segment descriptors and the search tree of the plan's forward tile size -
 * into a fixed array that the library holds in each GPU's memory from load to
 * process end (HP_STATIC_MAX_TABLE_BYTES, 64 KiB: about 1700 segments), and
 * launches the same kernel on them.  The table bytes travel as arguments of
 * small copy kernels on `stream` ahead of the transform kernel, so no host
 * buffer has to outlive the call.  It calls no hipMalloc / hipFree / hipMemcpy
 * and no other allocating routine.  The first call on a device looks up the
 * array's address (hipGetSymbolAddress); make that call outside graph capture.
 *   plan, src_bufs, dst_bufs, stream: as for hp_forward; the result is the same.
 * Returns HP_ELAYOUT when the tables exceed HP_STATIC_MAX_TABLE_BYTES (use
 * hp_forward with a device plan then), otherwise hp_forward's codes; HP_ESTATE
 * is not returned for host-only plans here.
 * All calls on one GPU share that GPU's array and it keeps the last call's
 * tables: calls on the SAME stream are ordered by the stream, calls that overlap
 * on different streams (or threads using different streams) of one GPU race on
 * it and must be serialised by the caller.  No timing events are attached. */
#define HP_STATIC_MAX_TABLE_BYTES 65536
int hp_forward_static(const hp_plan_t *plan, const void *const *src_bufs,
                      void *const *dst_bufs, void *stream);

/* Launch shape of one direction of a plan (direction 0 = hp_forward,
 * 1 = hp_backward, 2 = hp_backward_accumulate).  A plan starts from the
 * process-wide defaults below (the accumulating backward from the backward
 * defaults, with tiles of at least 4 KiB when a tile size is set there), or
 * from what hp_plan_tune found earlier for the same problem class. */
typedef struct hp_launch {
    int32_t tile_bytes;      /* boundary bytes per workgroup: 1024 << k, k = 0..6              */
    int32_t block_threads;   /* workgroup size: multiple of 64 in [64, 1024]                   */
    int32_t waves_per_cu;    /* cap on resident waves per compute unit, 0 = none; both kernels
                                reach their best HBM rate well below full occupancy            */
    int32_t nontemporal;     /* bit 0 = streaming (non-temporal) loads, bit 1 = streaming stores */
} hp_launch_t;
int hp_plan_get_launch(const hp_plan_t *plan, int32_t direction, hp_launch_t *out);
int hp_plan_set_launch(hp_plan_t *plan, int32_t direction, const hp_launch_t *in);

/* Measures a set of launch shapes on the caller's real buffers and keeps the
 * fastest in the plan (tile size x workgroup size x resident-wave cap; the
 * best cap depends on the replica count and row size, and the optimum is
 * narrow).  Arguments as for hp_forward and hp_backward; pass both pointers of
 * a direction as NULL to leave that direction alone.  The candidate launches
 * compute exactly what hp_forward / hp_backward compute, so the buffers end up
 * as after one such call.  Candidates are timed as bursts of back-to-back
 * launches, so that work a shape leaves behind at the end of a kernel (dirty
 * lines still draining to HBM) is charged to it and not to the next kernel.
 * When the buffers of both directions are given, every candidate launch of one
 * direction is followed by a launch of the other direction with its current
 * shape, and the pair is what is timed: a shape is judged in the sequence
 * forward, backward, forward, ... rather than against copies of itself.
 * A plan whose hp_forward launch moves less than 1 GiB keeps its shapes (it
 * still gets one launch per given direction): a timing loop over so little data
 * runs out of the 256 MB memory-side cache and would rank shapes by a behaviour
 * that a training step's fresh buffers do not show.
 * SYNCHRONOUS: waits on `stream` repeatedly, takes tens to hundreds of
 * milliseconds, creates and destroys four HIP events, and must not run
 * concurrently with other calls that use the same plan.
 * The winning shapes are also remembered per problem class (dtype, row size,
 * TP_dst copies, TP_src copies, device): plans of the same class created later
 * by hp_plan_create / hp_plan_create_batched / hp_plan_create_joined start from them instead of the
 * process-wide defaults, so a caller that rebuilds its plan every step tunes
 * once.  hp_forget_tuned_shapes drops what was remembered. */
int hp_plan_tune(hp_plan_t *plan, const void *const *src_bufs, void *const *dst_bufs,
                 const void *const *dst_grad_bufs, void *const *src_grad_bufs, void *stream);
void hp_forget_tuned_shapes(void);

/* The same search for hp_backward_accumulate (direction 2).  Every candidate
 * launch ADDS the folded gradients to src_accum_bufs, an unspecified number of
 * times in total: pass scratch accumulators of the right shape, not live ones.
 * Otherwise as hp_plan_tune. */
int hp_plan_tune_accumulate(hp_plan_t *plan, const void *const *dst_grad_bufs,
                            void *const *src_accum_bufs, void *stream);

/* Process-wide defaults copied into every plan created afterwards (integers).
 * Keys: "tile_bytes_fwd", "tile_bytes_bwd", "block_threads_fwd",
 * "block_threads_bwd", "waves_per_cu_fwd", "waves_per_cu_bwd",
 * "nontemporal_fwd", "nontemporal_bwd"; meanings and ranges as in hp_launch_t.
 * The tile size, the workgroup size and the resident-wave cap also take HP_AUTO
 * (-1, their initial value): the plan then picks them from its replica counts - the more buffers a
 * row's traffic spreads over (1 + TP_dst forward, TP_dst + TP_src backward) the
 * lower the cap, so that about 100 KB per compute unit stay in flight; the
 * figures are what hp_plan_tune finds most often per replica count.
 * Returns HP_EINVAL for an unknown key or an out-of-range value. */
#define HP_AUTO (-1)
int hp_set_option(const char *key, int64_t value);
int64_t hp_get_option(const char *key);     /* INT64_MIN for an unknown key */

/* Streaming probe for measurement harnesses: the HBM rate of a plain kernel
 * that reads n_read (0..8) linear arrays and writes n_write (0..8) linear arrays
 * (at least one array in all; n_write = 0 is a read-only stream whose data is
 * folded and dropped) of bytes_per_array bytes each, with the same 16-byte lanes, one-shot
 * workgroups and occupancy cap as the transform kernels but no segment lookup:
 * the practical ceiling of hp_forward's 1-read : TP_dst-write pattern and of
 * hp_backward's TP_dst-read : TP_src-write pattern on this machine.  With
 * shape == NULL it searches the launch shapes hp_plan_tune searches (one burst
 * each, then the best five again by the median of three bursts) and reports
 * the best (also in *best_shape if not NULL); otherwise it times the
 * given shape.  *gbps_out receives (n_read + n_write) * bytes / best time in
 * GB/s.  Allocates and frees its own device buffers, stream and events;
 * SYNCHRONOUS. */
int hp_probe_stream(int32_t n_read, int32_t n_write, int64_t bytes_per_array,
                    const hp_launch_t *shape, double *gbps_out, hp_launch_t *best_shape);

/* The same probe with a fixed launch shape (required) and another way of
 * handing tiles to workgroups, to show what the transform kernels' schedule
 * (HP_PROBE_ONESHOT) gains or loses against the alternatives on this machine:
 *   HP_PROBE_XCD_CHUNKED     one-shot workgroups, but the tile order is remapped
 *                            so that the workgroups landing on one of the 8 XCDs
 *                            (round-robin by workgroup id) walk one contiguous
 *                            eighth of every array;
 *   HP_PROBE_PERSISTENT      a grid of waves_per_cu / (block_threads / 64)
 *                            workgroups per compute unit (8 per unit when
 *                            waves_per_cu is 0); each workgroup loops over the
 *                            tiles with the grid size as stride;
 *   HP_PROBE_PERSISTENT_XCD  persistent, each XCD's workgroups stride through
 *                            their own contiguous eighth;
 *   HP_PROBE_PHASED          persistent, and a workgroup loads its whole tile
 *                            (4, 8 or 16 sixteen-byte chunks per lane, i.e.
 *                            tile_bytes = 64, 128 or 256 x block_threads) into
 *                            registers before its first store: reads and
 *                            writes reach HBM in long separate bursts
 *                            (n_read <= 1, n_write >= 1).
 * Otherwise as hp_probe_stream (allocates its own buffers, SYNCHRONOUS). */
#define HP_PROBE_ONESHOT        0
#define HP_PROBE_XCD_CHUNKED    1
#define HP_PROBE_PERSISTENT     2
#define HP_PROBE_PERSISTENT_XCD 3
#define HP_PROBE_PHASED         4
int hp_probe_stream_ex(int32_t n_read, int32_t n_write, int64_t bytes_per_array,
                       const hp_launch_t *shape, int32_t schedule, double *gbps_out);

/* Kernel timing for measurement harnesses.  hp_profile_enable(n) with n > 0
 * creates n HIP event pairs; from then on each hp_forward / hp_backward launch
 * (in call order, any thread) is stamped with the begin and end time of its own
 * kernel dispatch until the n pairs are used up; later launches are not timed.
 * n = 0 disables timing and frees the events.  hp_profile_read waits for the
 * recorded launches, writes their kernel durations in milliseconds to ms[] and
 * their kind (0 = hp_forward, 1 = hp_backward, 2 = hp_backward_accumulate) to
 * kinds[] (host arrays of `cap` entries), rewinds the recorder and returns the
 * number of launches recorded.  A launch that carries events goes through the
 * extended launch call and cannot be recorded into a HIP graph; with timing
 * disabled every launch is a plain kernel launch and can. */
int hp_profile_enable(int32_t max_launches);
int hp_profile_read(float *ms, int32_t *kinds, int32_t cap);

const char *hp_strerror(int code);
/* hipError_t value of the most recent failing HIP call on this thread (0 if none). */
int hp_last_hip_error(void);
const char *hp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HP_H_ */
