"""Host logic of the library, no GPU needed: the C ABI loads and exports what
include/hp.h declares, the plan builder's segment tables describe exactly the
row routing the oracle derives, and bad inputs come back as error codes."""
import ctypes as C
import os
import re
from dataclasses import replace

import numpy as np
import pytest

import paper_2605_27678_amd as hp
from oracle import oracle
from paper_2605_27678_amd import binding
from paper_2605_27678_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "hp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(hp_[a-z_0-9]+)\s*\(", text))
    assert {"hp_plan_create", "hp_forward", "hp_backward", "hp_plan_destroy"} <= declared
    L = C.CDLL(binding.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(L, name), name
    assert declared == set(binding.EXPORTS)
    assert "gfx950" in hp.hp_version()


def expand_segments(plan):
    """Per destination buffer: (src_buf, src_row) of every local row, -1 = text."""
    info = plan.info
    sb = -np.ones((info.n_dst_bufs, info.dst_rows_per_buf), np.int32)
    sr = -np.ones((info.n_dst_bufs, info.dst_rows_per_buf), np.int64)
    for s in plan.segments():
        rows = s.dst_row0 + s.dst_row_stride * np.arange(s.n_rows)
        for c in range(info.dst_copies):
            assert np.all(sb[s.dst_buf0 + c, rows] == -1)          # no row written twice
            sb[s.dst_buf0 + c, rows] = s.src_buf
            sr[s.dst_buf0 + c, rows] = s.src_row0 + np.arange(s.n_rows)
    return sb, sr


def check_against_oracle(src, dst, tm):
    plan = hp.hp_plan_create_host(src, dst, tm)
    prob = oracle.Problem(src, dst, tm)
    info = plan.info
    assert info.n_src_bufs == prob.n_src and info.n_dst_bufs == prob.n_dst
    assert plan.src_rows() == prob.src_rows()
    assert info.dst_rows_per_buf == prob.dst_rows()
    assert info.n_rows == tm.n_rows and info.row_bytes == 2 * tm.hidden
    assert info.boundary_bytes == tm.n_rows * tm.hidden * 2
    assert info.fwd_bytes == (1 + info.dst_copies) * info.boundary_bytes
    assert info.bwd_bytes == (info.dst_copies + info.src_copies) * info.boundary_bytes
    sb, sr = expand_segments(plan)
    for j in range(prob.n_dst):
        osb, osr = prob.forward_map(j)
        assert np.array_equal(sb[j], osb), j
        assert np.array_equal(sr[j], osr), j
    plan.close()
    return info


@pytest.mark.parametrize("seed", range(80))
def test_segments_match_oracle_walk_random_layouts(seed):
    rng = np.random.default_rng(seed)
    src, dst, tm = wl.random_layout_case(rng)
    check_against_oracle(src, dst, tm)
    if (tm.seq // dst.cp) % dst.tp == 0:
        check_against_oracle(src, replace(dst, tp_mode=wl.TP_SEQ_SHARD), tm)


@pytest.mark.parametrize("seed", range(20))
def test_segments_match_oracle_walk_spans_out_of_position_order(seed):
    rng = np.random.default_rng(300 + seed)
    src, dst, tm = wl.random_layout_case(rng)
    check_against_oracle(src, dst, wl.shuffle_spans(rng, tm))


@pytest.mark.parametrize("seed", range(30))
def test_segments_match_oracle_walk_wide_grids(seed):
    """CP up to 16, TP up to 16, hundreds of segments (search trees of two and
    three levels), sequence-sharded or replicated."""
    rng = np.random.default_rng(4000 + seed)
    src, dst, tm = wl.random_wide_case(rng)
    plan = hp.hp_plan_create_host(src, dst, tm)
    prob = oracle.Problem(src, dst, tm)
    assert plan.src_rows() == prob.src_rows() and plan.info.n_rows == tm.n_rows
    sb, sr = expand_segments(plan)
    for j in range(prob.n_dst):
        osb, osr = prob.forward_map(j)
        assert np.array_equal(sb[j], osb) and np.array_equal(sr[j], osr), j


@pytest.mark.parametrize("k", [1, 2, 7, 8, 9, 32])
def test_segments_match_oracle_walk_long_context_image_counts(k):
    """Fewer images than source ranks (empty ranks), exactly as many, one more,
    and the maximum of the long-context generator."""
    w = wl.scaled(wl.long_context(n_images=k), 8)
    info = check_against_oracle(w.src, w.dst, w.maps[0])
    assert sum(1 for r in hp.hp_plan_create_host(w.src, w.dst, w.maps[0]).src_rows() if r == 0) == max(0, 8 - k)
    assert 1 <= info.n_segments <= 3 * k


@pytest.mark.parametrize("name", ["tiny", "colocated4", "colocated4_dense", "long_context", "large_scale"])
def test_segments_match_oracle_walk_named_configs(name):
    w = wl.scaled(wl.CONFIGS[name](), 8)           # same spans and grids, small hidden
    info = check_against_oracle(w.src, w.dst, w.maps[0])
    assert 1 <= info.n_segments <= 3 * w.maps[0].n_images


def test_non_colocated_microbatches_and_contiguous_variant():
    w = wl.scaled(wl.non_colocated(n_microbatches=4), 8)
    for tm in w.maps:
        check_against_oracle(w.src, w.dst, tm)
        check_against_oracle(w.src, replace(w.dst, cp_split=wl.CP_CONTIGUOUS), tm)


def test_full_size_infos():
    w = wl.long_context()
    p = hp.hp_plan_create_host(w.src, w.dst, w.maps[0])
    assert p.info.row_bytes == 10240 and p.info.dst_rows_per_buf == 16384
    assert p.info.n_tiles >= p.info.boundary_bytes // p.get_launch(0)["tile_bytes"]
    w = wl.large_scale()
    p = hp.hp_plan_create_host(w.src, w.dst, w.maps[0])
    assert (p.info.n_src_bufs, p.info.n_dst_bufs, p.info.src_copies, p.info.dst_copies) == (32, 32, 2, 8)


def test_empty_map_is_a_valid_empty_plan():
    tm = wl.TokenMap(2, 16, 8, [], [], [])
    p = hp.hp_plan_create_host(wl.Grid(dp=2), wl.Grid(tp=2, cp=2), tm)
    assert p.info.n_rows == 0 and p.info.n_tiles == 0 and p.src_rows() == [0, 0]


def _code(src, dst, tm):
    with pytest.raises(hp.HpError) as e:
        hp.hp_plan_create_host(src, dst, tm)
    return e.value.code


def test_error_codes():
    ok = wl.TokenMap(2, 16, 8, [0, 1], [0, 4], [4, 4])
    g = wl.Grid()
    assert _code(wl.Grid(tp=0), g, ok) == binding.HP_EINVAL
    assert _code(g, wl.Grid(cp_split=7), ok) == binding.HP_EINVAL
    assert _code(g, wl.Grid(row_order=2), ok) == binding.HP_EINVAL
    assert _code(g, wl.Grid(tp_mode=5), ok) == binding.HP_EINVAL
    assert _code(g, g, replace(ok, hidden=0)) == binding.HP_EINVAL
    assert _code(wl.Grid(cp=2), g, ok) == binding.HP_ELAYOUT            # encoder has CP = 1
    assert _code(g, wl.Grid(dp=3), ok) == binding.HP_ELAYOUT            # batch % DP
    assert _code(g, wl.Grid(cp=3), ok) == binding.HP_ELAYOUT            # seq % CP
    assert _code(g, wl.Grid(cp=8, cp_split=wl.CP_ZIGZAG), replace(ok, seq=24)) == binding.HP_ELAYOUT
    assert _code(g, wl.Grid(tp=3, tp_mode=wl.TP_SEQ_SHARD), ok) == binding.HP_ELAYOUT
    assert _code(wl.Grid(dp=420), wl.Grid(tp=8, cp=4), ok) == binding.HP_ELAYOUT   # too many buffers
    assert _code(g, wl.Grid(tp=32), ok) == binding.HP_ELAYOUT
    bad = lambda **kw: replace(ok, **{k: np.array(v, np.int32) for k, v in kw.items()})
    assert _code(g, g, bad(img_start=[0, 14])) == binding.HP_EMAP        # runs past the end
    assert _code(g, g, bad(img_start=[-1, 4])) == binding.HP_EMAP
    assert _code(g, g, bad(img_len=[0, 4])) == binding.HP_EMAP
    assert _code(g, g, bad(img_sample=[0, 2])) == binding.HP_EMAP        # sample out of range
    assert _code(g, g, bad(img_sample=[1, 0])) == binding.HP_EMAP        # not in batch order
    assert _code(g, g, bad(img_sample=[0, 0], img_start=[0, 3])) == binding.HP_EMAP   # overlap
    assert _code(wl.Grid(dp=2), g, bad(img_src_dp=[1, 0])) == binding.HP_EMAP
    assert _code(wl.Grid(dp=2), g, bad(img_src_dp=[0, 2])) == binding.HP_EMAP
    # touching spans and out-of-order starts inside a sample are legal
    hp.hp_plan_create_host(g, g, bad(img_sample=[0, 0], img_start=[4, 0]))


def test_null_arguments_and_host_only_state():
    L = binding._lib()
    out = C.c_void_p(0)
    assert L.hp_plan_create_host(None, None, None, C.byref(out)) == binding.HP_EINVAL
    assert not out.value
    assert L.hp_plan_query(None, None) == binding.HP_EINVAL
    L.hp_plan_destroy(None)
    p = hp.hp_plan_create_host(wl.Grid(), wl.Grid(), wl.TokenMap(1, 4, 8, [0], [0], [4]))
    ptr = (C.c_void_p * 1)(C.c_void_p(64))
    assert L.hp_forward(p._h, ptr, ptr, None) == binding.HP_ESTATE      # no device tables
    assert L.hp_backward(p._h, ptr, ptr, None) == binding.HP_ESTATE
    assert L.hp_forward(p._h, None, ptr, None) == binding.HP_EINVAL
    assert b"token map" in L.hp_strerror(binding.HP_EMAP)
    assert L.hp_set_option(b"no_such_key", 1) == binding.HP_EINVAL
    assert L.hp_set_option(b"block_threads_fwd", 100) == binding.HP_EINVAL
    assert L.hp_set_option(b"tile_bytes_fwd", 3000) == binding.HP_EINVAL
    assert L.hp_set_option(b"tile_bytes_bwd", 131072) == binding.HP_EINVAL
    assert L.hp_set_option(b"waves_per_cu_bwd", 33) == binding.HP_EINVAL
    assert hp.hp_get_option("block_threads_fwd") in (-1, 64, 128, 256, 512, 1024)
    assert L.hp_set_option(b"block_threads_fwd", 0) == binding.HP_EINVAL
    assert L.hp_set_option(b"block_threads_fwd", -2) == binding.HP_EINVAL
    assert hp.hp_get_option("nope") == -2 ** 63
    assert L.hp_profile_enable(-1) == binding.HP_EINVAL
    assert L.hp_profile_enable(0) == binding.HP_OK
    assert L.hp_profile_read(None, None, 4) == binding.HP_EINVAL
    assert L.hp_profile_read(None, None, 0) == 0


def test_batched_plan_is_the_concatenation_of_its_microbatches():
    """A batched plan routes microbatch m exactly like the single plan of map m,
    with buffer indices shifted by m times the per-microbatch counts."""
    w = wl.scaled(wl.non_colocated(n_microbatches=5), 8)
    plan = hp.hp_plan_create_batched(w.src, w.dst, w.maps, host_only=True)
    n_src, n_dst = w.src.n_ranks, w.dst.n_ranks
    assert plan.info.n_maps == 5
    assert (plan.info.n_src_bufs, plan.info.n_dst_bufs) == (5 * n_src, 5 * n_dst)
    assert plan.info.n_rows == sum(m.n_rows for m in w.maps)
    sb, sr = expand_segments(plan)
    rows = plan.src_rows()
    for mi, tm in enumerate(w.maps):
        prob = oracle.Problem(w.src, w.dst, tm)
        assert rows[mi * n_src:(mi + 1) * n_src] == prob.src_rows()
        for j in range(n_dst):
            osb, osr = prob.forward_map(j)
            want = np.where(osb >= 0, osb + mi * n_src, -1)
            assert np.array_equal(sb[mi * n_dst + j], want)
            assert np.array_equal(sr[mi * n_dst + j], osr)
    # shapes must agree across microbatches; too many buffers is refused
    with pytest.raises(hp.HpError) as e:
        hp.hp_plan_create_batched(w.src, w.dst, [w.maps[0], replace(w.maps[1], hidden=16)], host_only=True)
    assert e.value.code == binding.HP_ELAYOUT
    with pytest.raises(hp.HpError) as e:
        hp.hp_plan_create_batched(w.src, w.dst, [w.maps[0]] * 60, host_only=True)
    assert e.value.code == binding.HP_ELAYOUT
    L = binding._lib()
    out = C.c_void_p(0)
    assert L.hp_plan_create_batched(None, None, None, 0, 1, C.byref(out)) == binding.HP_EINVAL


def test_launch_shape_get_set_and_tile_counts():
    w = wl.long_context()
    p = hp.hp_plan_create_host(w.src, w.dst, w.maps[0])
    segs = p.segments()
    for tile in (1024, 4096, 65536):
        p.set_launch(0, tile_bytes=tile)
        want = sum(-(-(s.n_rows * p.info.row_bytes) // tile) for s in segs)    # dense segments: ceil by bytes
        assert p.info.n_tiles == want
    p.set_launch(1, tile_bytes=2048, block_threads=128, waves_per_cu=6, nontemporal=1)
    assert p.get_launch(1) == dict(tile_bytes=2048, block_threads=128, waves_per_cu=6, nontemporal=1)
    for bad in (dict(tile_bytes=3000), dict(block_threads=96), dict(waves_per_cu=40), dict(nontemporal=4)):
        with pytest.raises(hp.HpError):
            p.set_launch(0, **bad)
    # row-strided segments: rows shorter than a tile are grouped, longer rows are cut into pieces
    tm = wl.TokenMap(2, 8, 600, [0, 1], [0, 2], [8, 5])
    q = hp.hp_plan_create_host(wl.Grid(), wl.Grid(row_order=wl.ROW_SBH), tm)
    assert all(s.dst_row_stride == 2 for s in q.segments())
    q.set_launch(0, tile_bytes=4096)                      # 3 rows of 1200 B per tile
    assert q.info.n_tiles == sum(-(-s.n_rows // 3) for s in q.segments())
    q.set_launch(0, tile_bytes=1024)                      # every row = 2 pieces (1024 + 176 B)
    assert q.info.n_tiles == sum(2 * s.n_rows for s in q.segments())
    L = binding._lib()
    assert L.hp_plan_tune(None, None, None, None, None, None) == binding.HP_EINVAL


# ---- joined plans: several source modules into one destination -----------------

def _joined_case(seed, n_edges=2, n_maps=2):
    rng = np.random.default_rng(seed)
    _, dst, tm0 = wl.random_layout_case(rng)
    srcs = [wl.Grid(tp=int(rng.choice([1, 2])), dp=int(rng.choice([1, 2, 3, 4])), rank_offset=8 * e)
            for e in range(n_edges)]
    maps = [[None] * n_maps for _ in range(n_edges)]
    for m in range(n_maps):
        _, _, tm = wl.random_layout_case(rng)
        # same shapes as microbatch 0, fresh spans
        lens = [[int(x) for x in rng.integers(1, 6, size=int(rng.integers(0, 4)))] for _ in range(tm0.batch)]
        lens = [l if sum(l) <= tm0.seq else [] for l in lens]
        tm = wl.token_map_from_lens(rng, tm0.batch, tm0.seq, tm0.hidden, lens) if any(lens) else \
            wl.TokenMap(tm0.batch, tm0.seq, tm0.hidden, [], [], [])
        for e, part in enumerate(wl.split_edges(rng, tm, n_edges)):
            maps[e][m] = part
    return srcs, dst, maps


@pytest.mark.parametrize("seed", range(30))
def test_joined_plan_is_the_union_of_its_edges(seed):
    """Segments, source rows and byte counts of a joined plan equal those of one
    batched plan per edge, with the source buffers listed edge by edge; and the
    row-by-row expansion equals the oracle's walk of every (edge, microbatch)."""
    n_edges, n_maps = 2 + seed % 2, 1 + seed % 3
    srcs, dst, maps = _joined_case(seed, n_edges, n_maps)
    joined = hp.hp_plan_create_joined(srcs, dst, maps, host_only=True)
    assert joined.info.n_edges == n_edges and joined.info.n_maps == n_maps
    per_edge = [hp.hp_plan_create_batched(srcs[e], dst, maps[e], host_only=True) for e in range(n_edges)]
    assert joined.src_rows() == [r for p in per_edge for r in p.src_rows()]
    assert joined.info.n_rows == sum(p.info.n_rows for p in per_edge)
    assert joined.info.fwd_bytes == sum(p.info.fwd_bytes for p in per_edge)
    assert joined.info.bwd_bytes == sum(p.info.bwd_bytes for p in per_edge)
    assert joined.info.bwd_accum_bytes == sum(p.info.bwd_accum_bytes for p in per_edge)
    want, base = [], 0
    for p in per_edge:
        want += [(s.src_buf + base, s.dst_buf0, s.src_row0, s.dst_row0, s.n_rows, s.dst_row_stride)
                 for s in p.segments()]
        base += p.info.n_src_bufs
    got = [(s.src_buf, s.dst_buf0, s.src_row0, s.dst_row0, s.n_rows, s.dst_row_stride) for s in joined.segments()]
    assert got == want
    # against the oracle: destination buffer j of microbatch m, as seen from every edge
    sb, sr = expand_segments(joined)
    n_dst = dst.tp * dst.cp * dst.dp
    base = 0
    seen = np.zeros_like(sb, dtype=bool)
    for e in range(n_edges):
        per_map = srcs[e].tp * srcs[e].dp
        for m in range(n_maps):
            prob = oracle.Problem(srcs[e], dst, maps[e][m])
            for j in range(n_dst):
                osb, osr = prob.forward_map(j)
                rows = osb >= 0
                assert np.array_equal(sb[m * n_dst + j][rows], osb[rows] + base + m * per_map)
                assert np.array_equal(sr[m * n_dst + j][rows], osr[rows])
                assert not seen[m * n_dst + j][rows].any()
                seen[m * n_dst + j][rows] = True
        base += per_map * n_maps
    assert np.array_equal(seen, sb >= 0)             # nothing beyond what the edges account for


def test_joined_plan_errors():
    dst = wl.Grid(tp=2, cp=2, cp_split=wl.CP_ZIGZAG)
    a = wl.TokenMap(1, 64, 8, [0, 0], [4, 30], [10, 6])
    b_ok = wl.TokenMap(1, 64, 8, [0], [14], [16])
    b_overlap = wl.TokenMap(1, 64, 8, [0], [13], [4])              # runs into a's first span
    b_hidden = wl.TokenMap(1, 64, 16, [0], [14], [16])
    srcs = [wl.Grid(dp=2), wl.Grid(tp=2, dp=1)]
    hp.hp_plan_create_joined(srcs, dst, [[a], [b_ok]], host_only=True).close()
    for maps, code in (([[a], [b_overlap]], binding.HP_EMAP), ([[a], [b_hidden]], binding.HP_ELAYOUT)):
        with pytest.raises(hp.HpError) as ei:
            hp.hp_plan_create_joined(srcs, dst, maps, host_only=True)
        assert ei.value.code == code
    with pytest.raises(ValueError):
        hp.hp_plan_create_joined(srcs, dst, [[a]], host_only=True)
    # too many buffers in total: 2 edges x dp 200 + 4 destination buffers
    big = [wl.Grid(dp=222), wl.Grid(dp=222)]
    empty = wl.TokenMap(1, 64, 8, [], [], [])
    hp.hp_plan_create_joined(big, dst, [[a], [empty]], host_only=True).close()      # 444 + 4 = 448: allowed
    with pytest.raises(hp.HpError) as ei:
        hp.hp_plan_create_joined([wl.Grid(dp=223), wl.Grid(dp=222)], dst, [[a], [empty]], host_only=True)
    assert ei.value.code == binding.HP_ELAYOUT


def test_default_launch_shapes_follow_the_replica_counts():
    """HP_AUTO: the resident-wave cap falls as a row's traffic spreads over more
    buffers; explicit options override field by field."""
    tm = wl.TokenMap(1, 64, 64, [0], [8], [16])
    caps_f, caps_b = [], []
    for tp in (1, 2, 4, 8, 16):
        p = hp.hp_plan_create_host(wl.Grid(), wl.Grid(tp=tp), tm)
        f, b, a = p.get_launch(0), p.get_launch(1), p.get_launch(2)
        assert (f["tile_bytes"], f["block_threads"]) == ((4096, 256) if tp == 2 else (2048, 64)) and f["nontemporal"] == 2
        assert b["tile_bytes"] in (1024, 2048) and b["nontemporal"] == 3
        assert 4 <= a["waves_per_cu"] <= 24 and a["tile_bytes"] == 2048
        caps_f.append(f["waves_per_cu"] * 2048 // f["tile_bytes"])          # workgroups of 2 KiB-equivalents per CU
        caps_b.append(b["waves_per_cu"] * b["tile_bytes"])
    assert caps_f == sorted(caps_f, reverse=True) and caps_f[0] > caps_f[-1]
    assert caps_b == sorted(caps_b, reverse=True)
    lc = hp.hp_plan_create_host(wl.Grid(dp=8), wl.Grid(tp=4, cp=8, cp_split=wl.CP_ZIGZAG),
                                wl.TokenMap(1, 64, 64, [0], [8], [16]))
    assert lc.get_launch(0) == dict(tile_bytes=2048, block_threads=64, waves_per_cu=12, nontemporal=2)
    assert lc.get_launch(1) == dict(tile_bytes=1024, block_threads=64, waves_per_cu=16, nontemporal=3)
    assert lc.get_launch(2) == dict(tile_bytes=2048, block_threads=64, waves_per_cu=11, nontemporal=3)
    caps_a = [hp.hp_plan_create_host(wl.Grid(tp=ts), wl.Grid(tp=td), tm).get_launch(2)["waves_per_cu"]
              for ts, td in ((1, 1), (1, 2), (1, 4), (2, 4), (2, 8), (2, 16))]       # 5, 6, 8, 12, 16, 24 streams
    assert caps_a == [13, 13, 11, 9, 7, 7]
    saved = {k: hp.hp_get_option(k) for k in ("tile_bytes_fwd", "waves_per_cu_bwd", "tile_bytes_bwd")}
    assert set(saved.values()) == {-1}
    try:
        hp.hp_set_option("tile_bytes_fwd", 8192)
        hp.hp_set_option("waves_per_cu_bwd", 0)
        hp.hp_set_option("tile_bytes_bwd", 1024)
        q = hp.hp_plan_create_host(wl.Grid(), wl.Grid(tp=8), tm)
        assert q.get_launch(0)["tile_bytes"] == 8192 and q.get_launch(0)["waves_per_cu"] == 5   # cap still automatic
        assert q.get_launch(1)["waves_per_cu"] == 0 and q.get_launch(1)["tile_bytes"] == 1024
        assert q.get_launch(2)["tile_bytes"] == 4096 and q.get_launch(2)["waves_per_cu"] == 0
        with pytest.raises(hp.HpError):
            hp.hp_set_option("tile_bytes_fwd", 3000)
        with pytest.raises(hp.HpError):
            hp.hp_set_option("waves_per_cu_fwd", -2)
    finally:
        for k, v in saved.items():
            hp.hp_set_option(k, v)


def test_size_limits():
    """Rows up to 16 MiB; at most 2^31 - 1 tiles of 1 KiB per launch (a 2 TiB boundary)."""
    g = wl.Grid()
    one_row = lambda hidden: wl.TokenMap(1, 4, hidden, [0], [1], [2])
    p = hp.hp_plan_create_host(g, wl.Grid(tp=2), one_row(1 << 23))           # 16 MiB rows
    assert p.info.row_bytes == 1 << 24 and p.info.n_tiles == 2 * (1 << 24) // p.get_launch(0)["tile_bytes"]
    assert _code(g, g, one_row((1 << 23) + 8)) == binding.HP_ELAYOUT
    assert _code(g, g, replace(one_row((1 << 22) + 4), dtype=wl.DT_F32)) == binding.HP_ELAYOUT
    big = wl.TokenMap(1, 1 << 20, 1 << 20, [0], [0], [1 << 20])              # 2 TiB boundary: one tile too many
    assert _code(g, g, big) == binding.HP_ELAYOUT
    ok = wl.TokenMap(1, 1 << 20, 1 << 20, [0], [0], [(1 << 20) - 1])
    q = hp.hp_plan_create_host(g, wl.Grid(cp=2, cp_split=wl.CP_ZIGZAG), ok)
    assert q.info.boundary_bytes == ((1 << 20) - 1) << 21 and q.info.n_segments == 3   # chunks 1 and 2 sit back to back on rank 1
    q.set_launch(0, tile_bytes=1024)
    assert q.info.n_tiles == q.info.boundary_bytes // 1024
    # 4096 all-image samples of 2^21 one-element rows are one contiguous run of 2^33 rows on both
    # sides; a segment descriptor counts rows in 32 bits, so the run is cut, not truncated
    B, S = 4096, 1 << 21
    huge = wl.TokenMap(B, S, 1, list(range(B)), [0] * B, [S] * B)
    r = hp.hp_plan_create_host(g, g, huge)
    segs = r.segments()
    assert r.info.n_rows == B * S == 1 << 33 and len(segs) >= 3
    assert all(0 < s.n_rows < 1 << 32 for s in segs) and sum(s.n_rows for s in segs) == 1 << 33
    row = 0
    for s in segs:                                   # the pieces follow each other without a gap
        assert (s.src_buf, s.dst_buf0, s.src_row0, s.dst_row0, s.dst_row_stride) == (0, 0, row, row, 1)
        row += s.n_rows
    r.set_launch(0, tile_bytes=1024)
    assert r.info.n_tiles == sum(-(-2 * s.n_rows // 1024) for s in segs)


def test_plan_builder_fuzz_under_sanitizers(tmp_path):
    """The host plan builder (pure C++) compiled with ASan + UBSan and driven with
    40000 random inputs, valid and invalid: no sanitizer report, every segment
    of every accepted plan inside its buffers."""
    import subprocess
    exe = tmp_path / "fuzz_plan"
    csrc = os.path.join(ROOT, "paper_2605_27678_amd", "csrc")

    def build(sanitizers):
        r = subprocess.run(["g++", "-std=c++17", "-O1", "-g", *sanitizers, "-fno-sanitize-recover=all",
                            "-I", os.path.join(ROOT, "include"), "-I", csrc, os.path.join(ROOT, "tests", "fuzz_plan.cpp"),
                            os.path.join(csrc, "hp_plan.cpp"), "-o", str(exe)], capture_output=True, text=True, timeout=300)
        assert r.returncode == 0, r.stderr

    build(["-fsanitize=address,undefined", "-static-libasan"])
    first = subprocess.run([str(exe), "11", "10"], capture_output=True, text=True, timeout=300)
    if first.returncode != 0 and "ASan runtime does not come first" in first.stderr:
        build(["-fsanitize=undefined"])              # another library is preloaded here: UBSan only
    for seed in (11, 12):
        r = subprocess.run([str(exe), str(seed), "20000"], capture_output=True, text=True, timeout=300)
        assert r.returncode == 0, r.stdout + r.stderr
        accepted = int(r.stdout.split()[1])
        assert accepted > 2000, r.stdout


def test_every_tile_of_every_launch_shape_stays_in_bounds(tmp_path):
    """The tile lookup the kernels run (csrc/hp_tile.hpp, shared host/device
    code) walked on the CPU under ASan + UBSan: for 300 random plans and all seven
    tile sizes the tiles partition the segments exactly and stay inside the
    source and destination buffers."""
    import subprocess
    exe = tmp_path / "walk_tiles"
    csrc = os.path.join(ROOT, "paper_2605_27678_amd", "csrc")

    def build(sanitizers):
        r = subprocess.run(["g++", "-std=c++17", "-O1", "-g", *sanitizers, "-fno-sanitize-recover=all", "-Wall",
                            "-Wno-unknown-pragmas", "-I", os.path.join(ROOT, "include"), "-I", csrc,
                            os.path.join(ROOT, "tests", "walk_tiles.cpp"), os.path.join(csrc, "hp_plan.cpp"),
                            "-o", str(exe)], capture_output=True, text=True, timeout=300)
        assert r.returncode == 0, r.stderr

    build(["-fsanitize=address,undefined", "-static-libasan"])
    first = subprocess.run([str(exe), "5", "2"], capture_output=True, text=True, timeout=300)
    if first.returncode != 0 and "ASan runtime does not come first" in first.stderr:
        build(["-fsanitize=undefined"])
    r = subprocess.run([str(exe), "21", "300"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout + r.stderr
    assert int(r.stdout.split()[3]) > 1000000, r.stdout


def test_plans_from_several_threads():
    """Host-only plan creation, queries and option changes from eight threads at
    once (the binding releases the GIL inside the library)."""
    import threading
    errors = []

    def work(seed):
        try:
            rng = np.random.default_rng(seed)
            for i in range(60):
                src, dst, tm = wl.random_layout_case(rng)
                p = hp.hp_plan_create_host(src, dst, tm)
                assert p.info.n_rows == tm.n_rows
                assert p.get_launch(0)["tile_bytes"] in (1024, 2048, 4096)
                hp.hp_set_option("tile_bytes_fwd", (1024, 2048, 4096, -1)[i % 4])
                p.close()
        except Exception as e:                      # noqa: BLE001 - reported below
            errors.append(repr(e))

    threads = [threading.Thread(target=work, args=(s,)) for s in range(8)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    hp.hp_set_option("tile_bytes_fwd", -1)
    assert not errors, errors
