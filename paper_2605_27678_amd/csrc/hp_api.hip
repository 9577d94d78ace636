// C ABI and gfx950 kernels of the boundary layout transform.
//
// Both kernels are HBM-bound row movers (no dense contraction anywhere, so no
// MFMA): one workgroup per tile of the plan's table, 16-byte lanes, every
// boundary byte read exactly once (forward) or every replica byte read exactly
// once (backward).  Forward stores each 16-byte chunk to all destination TP
// copies from registers; backward loads the chunk from all copies, folds them
// in binary32 in ascending tp order inside one lane (no cross-lane traffic is
// needed because a lane owns the same eight elements of every replica), rounds
// once to bf16 and stores to all source TP copies.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstdint>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "hp.h"
#include "hp_plan.hpp"

namespace {

thread_local int g_last_hip_error = 0;

inline bool hip_failed(hipError_t e) {
    if (e == hipSuccess) return false;
    g_last_hip_error = (int)e;
    return true;
}

// Device pointers of every buffer of a call, passed by value in the kernel
// argument segment: sources first, destinations from index n_src on.  Lookups
// use wave-uniform indices and become scalar loads.
struct BufTable {
    void *p[HP_MAX_BUFFERS];
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <typename V, bool NT>
__device__ __forceinline__ V ld(const V *p) {
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <typename V, bool NT>
__device__ __forceinline__ void st(V *p, V v) {
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

constexpr int kUnroll = 4;

// ---------------------------------------------------------------------------
// forward: tile of the source buffer -> the same bytes in NREP destination copies
// ---------------------------------------------------------------------------
template <typename V, int NREP, bool NTL, bool NTS>
__global__ void __launch_bounds__(1024)
hp_forward_kernel(const hp::Tile *__restrict__ tiles, const BufTable bufs,
                  const uint32_t dst_base, const uint32_t row_bytes, const uint32_t nrep_rt) {
    const hp::Tile t = tiles[blockIdx.x];
    const uint32_t nrep = NREP > 0 ? (uint32_t)NREP : nrep_rt;
    const char *src = (const char *)bufs.p[t.src_buf] + t.src_off;
    const uint32_t n = t.nbytes / (uint32_t)sizeof(V);
    const uint32_t step = blockDim.x;

    if (t.pitch_rows == 1) {
        for (uint32_t i0 = threadIdx.x; i0 < n; i0 += step * kUnroll) {
            V v[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const uint32_t i = i0 + u * step;
                if (i < n) v[u] = ld<V, NTL>((const V *)src + i);
            }
#pragma unroll 4
            for (uint32_t r = 0; r < nrep; ++r) {
                char *dst = (char *)bufs.p[dst_base + t.dst_buf0 + r] + t.dst_off;
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    const uint32_t i = i0 + u * step;
                    if (i < n) st<V, NTS>((V *)dst + i, v[u]);
                }
            }
        }
    } else {
        // row-strided destination ([S,B,H] order with several samples per rank)
        const uint64_t pitch = (uint64_t)t.pitch_rows * row_bytes;
        for (uint32_t i = threadIdx.x; i < n; i += step) {
            const uint32_t byte = i * (uint32_t)sizeof(V);
            const uint32_t row = byte / row_bytes;
            const uint32_t col = byte - row * row_bytes;
            const V v = ld<V, NTL>((const V *)(src + byte));
            for (uint32_t r = 0; r < nrep; ++r) {
                char *dst = (char *)bufs.p[dst_base + t.dst_buf0 + r] + t.dst_off;
                st<V, NTS>((V *)(dst + row * pitch + col), v);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// backward: NREP destination-gradient copies -> fp32 fold -> bf16 -> source copies
// ---------------------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// binary32 -> bf16 bits, round-to-nearest-even, NaN kept quiet
__device__ __forceinline__ uint32_t bf16_rne(float f) {
    const uint32_t u = __float_as_uint(f);
    const uint32_t rounded = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    const uint32_t nan = (u >> 16) | 0x40u;
    return ((u & 0x7fffffffu) > 0x7f800000u) ? nan : rounded;
}

// W = 32-bit words per lane chunk (4, 2 or 1); W == 0 means one bf16 per lane.
template <int W> struct Chunk { typedef uint32_t type __attribute__((ext_vector_type(W))); };
template <> struct Chunk<1> { typedef uint32_t type; };
template <> struct Chunk<0> { typedef uint16_t type; };

template <int W>
struct Fold {
    typedef typename Chunk<W>::type V;
    static constexpr int kElems = W == 0 ? 1 : 2 * W;
    float acc[kElems];

    __device__ __forceinline__ static uint32_t word(const V &v, int j) {
        if constexpr (W >= 2) return v[j];
        else return (uint32_t)v;
    }
    __device__ __forceinline__ void first(const V &v) {
        if constexpr (W == 0) acc[0] = bf16_lo(v);
        else {
#pragma unroll
            for (int j = 0; j < W; ++j) { acc[2 * j] = bf16_lo(word(v, j)); acc[2 * j + 1] = bf16_hi(word(v, j)); }
        }
    }
    __device__ __forceinline__ void add(const V &v) {
        if constexpr (W == 0) acc[0] = acc[0] + bf16_lo(v);
        else {
#pragma unroll
            for (int j = 0; j < W; ++j) {
                acc[2 * j] = acc[2 * j] + bf16_lo(word(v, j));
                acc[2 * j + 1] = acc[2 * j + 1] + bf16_hi(word(v, j));
            }
        }
    }
    __device__ __forceinline__ V result() const {
        if constexpr (W == 0) return (uint16_t)bf16_rne(acc[0]);
        else if constexpr (W == 1) return bf16_rne(acc[0]) | (bf16_rne(acc[1]) << 16);
        else {
            V out;
#pragma unroll
            for (int j = 0; j < W; ++j) out[j] = bf16_rne(acc[2 * j]) | (bf16_rne(acc[2 * j + 1]) << 16);
            return out;
        }
    }
};

constexpr int kBwdUnroll = 2;

template <int W, int NREP, bool NTL, bool NTS>
__global__ void __launch_bounds__(1024)
hp_backward_kernel(const hp::Tile *__restrict__ tiles, const BufTable bufs,
                   const uint32_t dst_base, const uint32_t row_bytes,
                   const uint32_t nrep_rt, const uint32_t src_copies) {
    typedef typename Chunk<W>::type V;
    const hp::Tile t = tiles[blockIdx.x];
    const uint32_t nrep = NREP > 0 ? (uint32_t)NREP : nrep_rt;
    const uint32_t n = t.nbytes / (uint32_t)sizeof(V);
    const uint32_t step = blockDim.x;
    const uint64_t pitch = (uint64_t)t.pitch_rows * row_bytes;
    const bool dense = t.pitch_rows == 1;

    for (uint32_t i0 = threadIdx.x; i0 < n; i0 += step * kBwdUnroll) {
        Fold<W> f[kBwdUnroll];
        uint64_t goff[kBwdUnroll];
#pragma unroll
        for (int u = 0; u < kBwdUnroll; ++u) {
            const uint32_t i = i0 + u * step;
            const uint32_t byte = i * (uint32_t)sizeof(V);
            if (dense) goff[u] = byte;
            else {
                const uint32_t row = byte / row_bytes;
                goff[u] = row * pitch + (byte - row * row_bytes);
            }
        }
        // ascending tp: copy 0 starts the accumulator, copies 1.. are added in order
#pragma unroll 4
        for (uint32_t r = 0; r < nrep; ++r) {
            const char *g = (const char *)bufs.p[dst_base + t.dst_buf0 + r] + t.dst_off;
#pragma unroll
            for (int u = 0; u < kBwdUnroll; ++u) {
                const uint32_t i = i0 + u * step;
                if (i < n) {
                    const V v = ld<V, NTL>((const V *)(g + goff[u]));
                    if (r == 0) f[u].first(v); else f[u].add(v);
                }
            }
        }
        for (uint32_t s = 0; s < src_copies; ++s) {
            char *out = (char *)bufs.p[t.src_buf + s] + t.src_off;
#pragma unroll
            for (int u = 0; u < kBwdUnroll; ++u) {
                const uint32_t i = i0 + u * step;
                if (i < n) st<V, NTS>((V *)out + i, f[u].result());
            }
        }
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------

// Largest chunk width in {16, 8, 4, 2} bytes that divides the row size and
// every pointer the launch will touch.
int pick_width(const hp_plan *p, const BufTable &bt, int n_ptrs) {
    uint64_t bits = (uint64_t)p->row_bytes;
    for (int i = 0; i < n_ptrs; ++i) bits |= (uint64_t)(uintptr_t)bt.p[i];
    if ((bits & 15) == 0) return 16;
    if ((bits & 7) == 0) return 8;
    if ((bits & 3) == 0) return 4;
    if ((bits & 1) == 0) return 2;
    return 0;
}

// Optional per-launch kernel timing.  When enabled, every launch is given its own
// pair of HIP events through hipExtLaunchKernelGGL, which stamps them with the
// dispatch's own begin and end times (no extra marker packets in the stream, so
// the timed work is not perturbed).
struct Profiler {
    std::mutex mu;
    std::vector<hipEvent_t> start, stop;
    std::vector<int32_t> kind;
    size_t used = 0;
    bool enabled = false;
} g_prof;

struct EventPair { hipEvent_t start = nullptr, stop = nullptr; };

EventPair next_event_pair(int kind) {
    EventPair e;
    if (!g_prof.enabled) return e;
    std::lock_guard<std::mutex> lk(g_prof.mu);
    if (g_prof.enabled && g_prof.used < g_prof.start.size()) {
        e.start = g_prof.start[g_prof.used];
        e.stop = g_prof.stop[g_prof.used];
        g_prof.kind[g_prof.used] = kind;
        ++g_prof.used;
    }
    return e;
}

#define HP_LAUNCH(kind, kernel, grid, blk, lds, st, ...)                                        \
    do {                                                                                        \
        const EventPair ev_ = next_event_pair(kind);                                            \
        hipExtLaunchKernelGGL(kernel, grid, blk, lds, st, ev_.start, ev_.stop, 0, __VA_ARGS__); \
    } while (0)

struct LaunchCfg {
    unsigned block;      // threads per workgroup
    unsigned lds_bytes;  // dynamic LDS requested only to cap the workgroups resident per CU
};

// Both kernels run fastest well below full occupancy: with every wave slot
// busy the in-flight window of addresses is wide and HBM efficiency drops.  The
// cap is expressed in waves per CU and enforced by requesting a slice of the
// CU's 160 KB LDS per workgroup (the kernels do not touch it).
LaunchCfg launch_cfg(int64_t block, int64_t waves_per_cu) {
    LaunchCfg c{(unsigned)block, 0u};
    const int64_t waves_per_wg = block / 64;
    if (waves_per_cu > 0) {
        int64_t wgs = waves_per_cu / waves_per_wg;
        if (wgs < 2) wgs = 2;
        if (wgs < 32) {
            int64_t lds = (160 * 1024) / wgs - 512;
            lds = lds / 512 * 512;
            if (lds > 64 * 1024) lds = 64 * 1024;
            c.lds_bytes = (unsigned)lds;
        }
    }
    return c;
}

template <typename V, bool NTL, bool NTS>
void launch_forward_nrep(const hp_plan *p, const BufTable &bt, hipStream_t st, LaunchCfg c) {
    const dim3 grid((unsigned)p->tiles.size()), blk(c.block);
    const uint32_t base = (uint32_t)p->n_src_bufs, rb = (uint32_t)p->row_bytes, nrep = (uint32_t)p->dst_copies;
    switch (p->dst_copies) {
        case 1: HP_LAUNCH(0, (hp_forward_kernel<V, 1, NTL, NTS>), grid, blk, c.lds_bytes, st, p->d_tiles, bt, base, rb, nrep); break;
        case 2: HP_LAUNCH(0, (hp_forward_kernel<V, 2, NTL, NTS>), grid, blk, c.lds_bytes, st, p->d_tiles, bt, base, rb, nrep); break;
        case 4: HP_LAUNCH(0, (hp_forward_kernel<V, 4, NTL, NTS>), grid, blk, c.lds_bytes, st, p->d_tiles, bt, base, rb, nrep); break;
        case 8: HP_LAUNCH(0, (hp_forward_kernel<V, 8, NTL, NTS>), grid, blk, c.lds_bytes, st, p->d_tiles, bt, base, rb, nrep); break;
        default: HP_LAUNCH(0, (hp_forward_kernel<V, 0, NTL, NTS>), grid, blk, c.lds_bytes, st, p->d_tiles, bt, base, rb, nrep); break;
    }
}

template <bool NTL, bool NTS>
void launch_forward(const hp_plan *p, const BufTable &bt, hipStream_t st, LaunchCfg c, int width) {
    switch (width) {
        case 16: launch_forward_nrep<u32x4, NTL, NTS>(p, bt, st, c); break;
        case 8: launch_forward_nrep<u32x2, NTL, NTS>(p, bt, st, c); break;
        case 4: launch_forward_nrep<uint32_t, NTL, NTS>(p, bt, st, c); break;
        default: launch_forward_nrep<uint16_t, NTL, NTS>(p, bt, st, c); break;
    }
}

template <int W, bool NTL, bool NTS>
void launch_backward_nrep(const hp_plan *p, const BufTable &bt, hipStream_t st, LaunchCfg c) {
    const dim3 grid((unsigned)p->tiles.size()), blk(c.block);
    const uint32_t base = (uint32_t)p->n_src_bufs, rb = (uint32_t)p->row_bytes;
    const uint32_t nrep = (uint32_t)p->dst_copies, sc = (uint32_t)p->src_copies;
    switch (p->dst_copies) {
        case 1: HP_LAUNCH(1, (hp_backward_kernel<W, 1, NTL, NTS>), grid, blk, c.lds_bytes, st, p->d_tiles, bt, base, rb, nrep, sc); break;
        case 2: HP_LAUNCH(1, (hp_backward_kernel<W, 2, NTL, NTS>), grid, blk, c.lds_bytes, st, p->d_tiles, bt, base, rb, nrep, sc); break;
        case 4: HP_LAUNCH(1, (hp_backward_kernel<W, 4, NTL, NTS>), grid, blk, c.lds_bytes, st, p->d_tiles, bt, base, rb, nrep, sc); break;
        case 8: HP_LAUNCH(1, (hp_backward_kernel<W, 8, NTL, NTS>), grid, blk, c.lds_bytes, st, p->d_tiles, bt, base, rb, nrep, sc); break;
        default: HP_LAUNCH(1, (hp_backward_kernel<W, 0, NTL, NTS>), grid, blk, c.lds_bytes, st, p->d_tiles, bt, base, rb, nrep, sc); break;
    }
}

template <bool NTL, bool NTS>
void launch_backward(const hp_plan *p, const BufTable &bt, hipStream_t st, LaunchCfg c, int width) {
    switch (width) {
        case 16: launch_backward_nrep<4, NTL, NTS>(p, bt, st, c); break;
        case 8: launch_backward_nrep<2, NTL, NTS>(p, bt, st, c); break;
        case 4: launch_backward_nrep<1, NTL, NTS>(p, bt, st, c); break;
        default: launch_backward_nrep<0, NTL, NTS>(p, bt, st, c); break;
    }
}

// Fills the pointer table and checks what the kernels assume: every buffer a
// tile touches is present, and the plan's tables live on the current device.
// `read_all_src` is false for forward (only copy tp = 0 of a source rank is
// read) and true for backward (every copy is written).
int prepare(const hp_plan *p, const void *const *src, const void *const *dst, bool all_src_copies,
            BufTable *bt, int *width) {
    if (!p || !src || !dst) return HP_EINVAL;
    if (!p->d_tiles && !p->tiles.empty()) return HP_ESTATE;
    int dev = -1;
    if (!p->tiles.empty()) {
        if (hip_failed(hipGetDevice(&dev))) return HP_EHIP;
        if (dev != p->device) return HP_ESTATE;
    }
    std::memset(bt, 0, sizeof(*bt));
    int n = 0;
    for (int i = 0; i < p->n_src_bufs; ++i) {
        const bool needed = p->src_rows[i] > 0 && (all_src_copies || i % p->src_copies == 0);
        if (needed && !src[i]) return HP_EINVAL;
        bt->p[n++] = needed ? const_cast<void *>(src[i]) : nullptr;
    }
    for (int j = 0; j < p->n_dst_bufs; ++j) {
        if (!dst[j] && p->n_rows > 0) return HP_EINVAL;
        bt->p[n++] = const_cast<void *>(dst[j]);
    }
    *width = pick_width(p, *bt, n);
    if (*width == 0) return HP_EALIGN;
    return HP_OK;
}

int finish_launch() {
    if (hip_failed(hipGetLastError())) return HP_EHIP;
    return HP_OK;
}

int create_common(const hp_layout_t *src, const hp_layout_t *dst, const hp_token_map_t *map,
                  bool upload, hp_plan_t **out) {
    if (!out) return HP_EINVAL;
    hp_plan *p = new (std::nothrow) hp_plan();
    if (!p) return HP_ENOMEM;
    int rc;
    try {
        rc = hp::build_host_plan(src, dst, map, p);
    } catch (const std::bad_alloc &) {
        rc = HP_ENOMEM;
    } catch (...) {
        rc = HP_EINVAL;
    }
    if (rc == HP_OK && upload) {
        if (hip_failed(hipGetDevice(&p->device))) rc = HP_EHIP;
        if (rc == HP_OK && !p->tiles.empty()) {
            const size_t bytes = p->tiles.size() * sizeof(hp::Tile);
            hipError_t e = hipMalloc((void **)&p->d_tiles, bytes);
            if (e == hipErrorOutOfMemory) { g_last_hip_error = (int)e; rc = HP_ENOMEM; }
            else if (hip_failed(e)) rc = HP_EHIP;
            if (rc == HP_OK && hip_failed(hipMemcpy(p->d_tiles, p->tiles.data(), bytes, hipMemcpyHostToDevice)))
                rc = HP_EHIP;
        }
    }
    if (rc != HP_OK) {
        if (p->d_tiles) (void)hipFree(p->d_tiles);
        delete p;
        return rc;
    }
    *out = p;
    return HP_OK;
}

struct OptionDesc {
    const char *name;
    int64_t hp::Options::*field;
    int64_t lo, hi, multiple;
};
const OptionDesc kOptions[] = {
    {"tile_bytes", &hp::Options::tile_bytes, 256, 1 << 24, 1},
    {"block_threads_fwd", &hp::Options::block_threads_fwd, 64, 1024, 64},
    {"block_threads_bwd", &hp::Options::block_threads_bwd, 64, 1024, 64},
    {"nontemporal_fwd", &hp::Options::nontemporal_fwd, 0, 3, 1},
    {"nontemporal_bwd", &hp::Options::nontemporal_bwd, 0, 3, 1},
    {"waves_per_cu_fwd", &hp::Options::waves_per_cu_fwd, 0, 32, 1},
    {"waves_per_cu_bwd", &hp::Options::waves_per_cu_bwd, 0, 32, 1},
};

}  // namespace

extern "C" {

int hp_plan_create(const hp_layout_t *src, const hp_layout_t *dst, const hp_token_map_t *map,
                   hp_plan_t **out) {
    return create_common(src, dst, map, true, out);
}

int hp_plan_create_host(const hp_layout_t *src, const hp_layout_t *dst, const hp_token_map_t *map,
                        hp_plan_t **out) {
    return create_common(src, dst, map, false, out);
}

void hp_plan_destroy(hp_plan_t *plan) {
    if (!plan) return;
    if (plan->d_tiles) (void)hipFree(plan->d_tiles);
    delete plan;
}

int hp_plan_query(const hp_plan_t *p, hp_plan_info_t *info) {
    if (!p || !info) return HP_EINVAL;
    hp_plan_info_t o;
    std::memset(&o, 0, sizeof(o));
    o.n_src_bufs = p->n_src_bufs;
    o.n_dst_bufs = p->n_dst_bufs;
    o.src_copies = p->src_copies;
    o.dst_copies = p->dst_copies;
    o.n_rows = p->n_rows;
    o.row_bytes = p->row_bytes;
    o.dst_rows_per_buf = p->dst_rows_per_buf;
    o.boundary_bytes = p->n_rows * p->row_bytes;
    o.fwd_bytes = (1 + (int64_t)p->dst_copies) * o.boundary_bytes;
    o.bwd_bytes = ((int64_t)p->dst_copies + p->src_copies) * o.boundary_bytes;
    o.n_segments = (int32_t)p->segments.size();
    o.n_tiles = (int32_t)p->tiles.size();
    o.on_device = (p->d_tiles != nullptr || (p->device >= 0 && p->tiles.empty())) ? 1 : 0;
    o.device = p->device;
    *info = o;
    return HP_OK;
}

int hp_plan_src_rows(const hp_plan_t *p, int64_t *rows, int32_t cap) {
    if (!p || (!rows && cap > 0) || cap < 0) return HP_EINVAL;
    for (int32_t i = 0; i < p->n_src_bufs && i < cap; ++i) rows[i] = p->src_rows[i];
    return p->n_src_bufs;
}

int hp_plan_segments(const hp_plan_t *p, hp_segment_t *out, int32_t cap) {
    if (!p || (!out && cap > 0) || cap < 0) return HP_EINVAL;
    const int32_t n = (int32_t)p->segments.size();
    for (int32_t i = 0; i < n && i < cap; ++i) out[i] = p->segments[i];
    return n;
}

int hp_forward(const hp_plan_t *p, const void *const *src_bufs, void *const *dst_bufs, void *stream) {
    BufTable bt;
    int width = 0;
    int rc = prepare(p, src_bufs, (const void *const *)dst_bufs, false, &bt, &width);
    if (rc != HP_OK) return rc;
    if (p->tiles.empty()) return HP_OK;
    const LaunchCfg block = launch_cfg(hp::options().block_threads_fwd, hp::options().waves_per_cu_fwd);
    switch (hp::options().nontemporal_fwd & 3) {
        case 0: launch_forward<false, false>(p, bt, (hipStream_t)stream, block, width); break;
        case 1: launch_forward<true, false>(p, bt, (hipStream_t)stream, block, width); break;
        case 2: launch_forward<false, true>(p, bt, (hipStream_t)stream, block, width); break;
        default: launch_forward<true, true>(p, bt, (hipStream_t)stream, block, width); break;
    }
    return finish_launch();
}

int hp_backward(const hp_plan_t *p, const void *const *dst_grad_bufs, void *const *src_grad_bufs,
                void *stream) {
    BufTable bt;
    int width = 0;
    int rc = prepare(p, (const void *const *)src_grad_bufs, dst_grad_bufs, true, &bt, &width);
    if (rc != HP_OK) return rc;
    if (p->tiles.empty()) return HP_OK;
    const LaunchCfg block = launch_cfg(hp::options().block_threads_bwd, hp::options().waves_per_cu_bwd);
    switch (hp::options().nontemporal_bwd & 3) {
        case 0: launch_backward<false, false>(p, bt, (hipStream_t)stream, block, width); break;
        case 1: launch_backward<true, false>(p, bt, (hipStream_t)stream, block, width); break;
        case 2: launch_backward<false, true>(p, bt, (hipStream_t)stream, block, width); break;
        default: launch_backward<true, true>(p, bt, (hipStream_t)stream, block, width); break;
    }
    return finish_launch();
}

int hp_set_option(const char *key, int64_t value) {
    if (!key) return HP_EINVAL;
    for (const OptionDesc &d : kOptions) {
        if (std::strcmp(key, d.name)) continue;
        if (value < d.lo || value > d.hi || (d.multiple > 1 && value % d.multiple)) return HP_EINVAL;
        hp::options().*(d.field) = value;
        return HP_OK;
    }
    return HP_EINVAL;
}

int64_t hp_get_option(const char *key) {
    if (key)
        for (const OptionDesc &d : kOptions)
            if (!std::strcmp(key, d.name)) return hp::options().*(d.field);
    return INT64_MIN;
}

int hp_profile_enable(int32_t max_launches) {
    if (max_launches < 0 || max_launches > (1 << 20)) return HP_EINVAL;
    std::lock_guard<std::mutex> lk(g_prof.mu);
    g_prof.enabled = false;
    for (hipEvent_t e : g_prof.start) (void)hipEventDestroy(e);
    for (hipEvent_t e : g_prof.stop) (void)hipEventDestroy(e);
    g_prof.start.clear(); g_prof.stop.clear(); g_prof.kind.clear();
    g_prof.used = 0;
    if (max_launches == 0) return HP_OK;
    try {
        g_prof.start.reserve(max_launches); g_prof.stop.reserve(max_launches);
        g_prof.kind.assign(max_launches, 0);
    } catch (const std::bad_alloc &) {
        return HP_ENOMEM;
    }
    for (int32_t i = 0; i < max_launches; ++i) {
        hipEvent_t a = nullptr, b = nullptr;
        if (hip_failed(hipEventCreate(&a)) || hip_failed(hipEventCreate(&b))) {
            if (a) (void)hipEventDestroy(a);
            for (hipEvent_t e : g_prof.start) (void)hipEventDestroy(e);
            for (hipEvent_t e : g_prof.stop) (void)hipEventDestroy(e);
            g_prof.start.clear(); g_prof.stop.clear(); g_prof.kind.clear();
            return HP_EHIP;
        }
        g_prof.start.push_back(a); g_prof.stop.push_back(b);
    }
    g_prof.enabled = true;
    return HP_OK;
}

int hp_profile_read(float *ms, int32_t *kinds, int32_t cap) {
    if (cap < 0 || (cap > 0 && (!ms || !kinds))) return HP_EINVAL;
    std::lock_guard<std::mutex> lk(g_prof.mu);
    const int32_t n = (int32_t)g_prof.used;
    for (int32_t i = 0; i < n && i < cap; ++i) {
        if (hip_failed(hipEventSynchronize(g_prof.stop[i]))) return HP_EHIP;
        float t = 0.f;
        if (hip_failed(hipEventElapsedTime(&t, g_prof.start[i], g_prof.stop[i]))) return HP_EHIP;
        ms[i] = t;
        kinds[i] = g_prof.kind[i];
    }
    g_prof.used = 0;
    return n;
}

const char *hp_strerror(int code) {
    switch (code) {
        case HP_OK: return "ok";
        case HP_EINVAL: return "invalid argument (null pointer, non-positive size or unknown enum)";
        case HP_ELAYOUT: return "grids do not divide the token map or exceed a library limit";
        case HP_EMAP: return "bad token map (span out of range, overlap, or unordered samples/ranks)";
        case HP_ENOMEM: return "out of memory";
        case HP_EHIP: return "HIP runtime error";
        case HP_ESTATE: return "plan has no device tables on the current device";
        case HP_EALIGN: return "buffer pointer not aligned to the element size";
        default: return "unknown error code";
    }
}

int hp_last_hip_error(void) { return g_last_hip_error; }

const char *hp_version(void) { return "hp-boundary 0.1 (gfx950)"; }

}  // extern "C"
