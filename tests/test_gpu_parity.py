"""GPU parity: hp_forward / hp_backward through the C ABI against the CPU
oracle, bit for bit.  Forward is a byte mover, so any difference is an error;
backward follows the same ascending-tp binary32 fold as the oracle, so it must
match bit for bit as well (NaN payloads excepted)."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import paper_2605_27678_amd as hp
from oracle import oracle
from paper_2605_27678_amd import workloads as wl
from parity import _to_host_bits, check_case, check_case_extended, make_inputs

pytestmark = pytest.mark.gpu

OPTION_KEYS = ("tile_bytes_fwd", "tile_bytes_bwd", "block_threads_fwd", "block_threads_bwd",
               "nontemporal_fwd", "nontemporal_bwd", "waves_per_cu_fwd", "waves_per_cu_bwd")


@pytest.fixture(autouse=True)
def _default_options():
    saved = {k: hp.hp_get_option(k) for k in OPTION_KEYS}
    yield
    for k, v in saved.items():
        hp.hp_set_option(k, v)
    hp.hp_forget_tuned_shapes()


def test_tiny_config():
    w = wl.tiny()
    info = check_case(w.src, w.dst, w.maps[0], seed=1)
    assert info.n_rows == 128 and info.on_device == 1


@pytest.mark.parametrize("seed", range(40))
def test_random_small_layouts(seed):
    """Random grids, both split rules, both row orders (strided path), explicit
    and default image placement, empty source ranks, hidden 8/16/24."""
    rng = np.random.default_rng(seed)
    src, dst, tm = wl.random_layout_case(rng)
    check_case(src, dst, tm, seed=seed)
    if (tm.seq // dst.cp) % dst.tp == 0:
        check_case(src, replace(dst, tp_mode=wl.TP_SEQ_SHARD), tm, seed=seed + 100)


@pytest.mark.parametrize("seed", range(10))
def test_spans_out_of_position_order(seed):
    """Images of a sample placed in the sequence in a shuffled order."""
    rng = np.random.default_rng(400 + seed)
    src, dst, tm = wl.random_layout_case(rng)
    check_case(src, dst, wl.shuffle_spans(rng, tm), seed=seed)


@pytest.mark.parametrize("seed", list(range(14)) + [50])          # seed 50: 404 segments, three tree levels
def test_random_wide_grids(seed):
    """CP up to 16, destination TP up to 16 (run-time replica counts 5 and 16),
    hundreds of segments: search trees of two and three levels; 1 KiB tiles so
    that most segments span several tiles with ragged ends."""
    from parity import check_case_extended
    rng = np.random.default_rng(4100 + seed)
    src, dst, tm = wl.random_wide_case(rng)
    hp.hp_set_option("tile_bytes_fwd", 1024)
    hp.hp_set_option("tile_bytes_bwd", 1024)
    check_case(src, dst, tm, seed=seed)
    if seed % 2:
        check_case_extended(src, dst, replace(tm, dtype=wl.DT_F32), seed=seed)
    else:
        check_case_extended(src, dst, tm, seed=seed)


@pytest.mark.parametrize("k", [1, 2, 7, 8, 9, 32])
def test_long_context_image_counts(k):
    """Config-3 grid with 1..32 images: empty source ranks when k < 8."""
    w = wl.scaled(wl.long_context(n_images=k), 320)
    check_case(w.src, w.dst, w.maps[0], seed=k)


@pytest.mark.parametrize("hidden", [7, 9, 12, 100, 320, 1000, 5120])
def test_long_context_spans_at_several_hidden_sizes(hidden):
    """The full config-3 grid and spans (34 segments, ragged tails, spans that
    straddle zigzag chunk borders) with rows of 14 B .. 10 KB: exercises the
    2/4/8/16-byte lane paths and many tiles per segment."""
    w = wl.long_context(n_images=9)
    tm = replace(w.maps[0], hidden=hidden)
    hp.hp_set_option("tile_bytes_fwd", 1024)
    hp.hp_set_option("tile_bytes_bwd", 2048)
    check_case(w.src, w.dst, tm, seed=hidden)


@pytest.mark.parametrize("tile,block,nt,waves", [(1024, 64, 1, 0), (1024, 128, 0, 4), (32768, 256, 2, 8),
                                                (65536, 512, 3, 16), (16384, 1024, 1, 32),
                                                (4096, 256, 2, 12), (2048, 64, 3, 1), (8192, 192, 0, 6)])
def test_launch_shapes(tile, block, nt, waves):
    hp.hp_set_option("tile_bytes_fwd", tile)
    hp.hp_set_option("tile_bytes_bwd", (1 << 26) // tile)          # 64 KiB .. 1 KiB, the other way round
    hp.hp_set_option("block_threads_fwd", block)
    hp.hp_set_option("block_threads_bwd", 64 * (16 // (block // 64)))
    hp.hp_set_option("waves_per_cu_fwd", waves)
    hp.hp_set_option("waves_per_cu_bwd", 32 - waves)
    hp.hp_set_option("nontemporal_fwd", nt)
    hp.hp_set_option("nontemporal_bwd", 3 - nt)
    w = wl.scaled(wl.large_scale(), 96)
    check_case(w.src, w.dst, w.maps[0], seed=tile % 97)


@pytest.mark.parametrize("tp", [1, 2, 3, 4, 5, 8, 16])
def test_replica_counts(tp):
    rng = np.random.default_rng(tp)
    tm = wl.token_map_from_lens(rng, 2, 96, 40, [[5, 17, 9], [30]])
    check_case(wl.Grid(tp=2, dp=3), wl.Grid(tp=tp, cp=2, dp=2, cp_split=wl.CP_ZIGZAG), tm, seed=tp)


def test_backward_order_and_special_values():
    """Wide dynamic range so that the order of the fold matters, plus inf, NaN,
    signed zeros and subnormals (binary32 subnormal sums must not be flushed)."""
    rng = np.random.default_rng(5)
    tm = wl.token_map_from_lens(rng, 1, 128, 64, [[20, 33, 7]])
    src, dst = wl.Grid(dp=2), wl.Grid(tp=4, cp=2, cp_split=wl.CP_ZIGZAG)
    prob = oracle.Problem(src, dst, tm)
    grads = []
    for j in range(prob.n_dst):
        e = rng.integers(-30, 30, size=(prob.dst_rows(), 64))
        x = (rng.standard_normal((prob.dst_rows(), 64)) * np.exp2(e)).astype(np.float32)
        t = torch.from_numpy(x).to(torch.bfloat16)
        bits = t.view(torch.int16)
        # sprinkle special patterns
        special = torch.tensor([0x7F80, -128, 0x7FC0, 0x0001, 0x0002, -32767, 0x0000, -32768, 0x007F, 0x0080],
                               dtype=torch.int16)     # -128 = 0xFF80 (-inf), -32767 = 0x8001, -32768 = 0x8000
        idx = torch.from_numpy(rng.integers(0, bits.numel(), size=400))
        bits.view(-1)[idx] = special[torch.from_numpy(rng.integers(0, len(special), size=400))]
        grads.append(t)
    # rows where all four replicas are subnormal
    for j in range(prob.n_dst):
        grads[j].view(torch.int16)[:, :4] = torch.from_numpy(
            rng.integers(1, 0x7F, size=(prob.dst_rows(), 4)).astype(np.int16))
    check_case(src, dst, tm, seed=3, grads_override=grads)


def test_order_sensitive_fixture_on_gpu():
    """[2^24, 1, -2^24, 1] summed ascending gives 1 (exact sum 2)."""
    tm = wl.TokenMap(1, 1, 8, [0], [0], [1])
    plan = hp.hp_plan_create(wl.Grid(), wl.Grid(tp=4), tm)
    vals = [16777216.0, 1.0, -16777216.0, 1.0]
    g = [torch.full((1, 8), v, dtype=torch.bfloat16, device="cuda") for v in vals]
    out = [torch.zeros((1, 8), dtype=torch.bfloat16, device="cuda")]
    hp.hp_backward(plan, g, out)
    torch.cuda.synchronize()
    assert out[0].float().cpu().tolist() == [[1.0] * 8]


def test_all_ones_returns_replica_count_and_text_rows_untouched():
    w = wl.scaled(wl.colocated4(), 64)
    tm = w.maps[0]
    plan = hp.hp_plan_create(w.src, w.dst, tm)
    rows = plan.src_rows()
    ones = [torch.ones((plan.info.dst_rows_per_buf, 64), dtype=torch.bfloat16, device="cuda") for _ in range(4)]
    sg = [torch.zeros((r, 64), dtype=torch.bfloat16, device="cuda") for r in rows]
    hp.hp_backward(plan, ones, sg)
    torch.cuda.synchronize()
    for t in sg:
        assert bool((t == 4.0).all())
    # forward of ones into a zero sequence marks exactly the image rows
    srcs = [torch.ones((r, 64), dtype=torch.bfloat16, device="cuda") for r in rows]
    dst = [torch.zeros((plan.info.dst_rows_per_buf, 64), dtype=torch.bfloat16, device="cuda") for _ in range(4)]
    hp.hp_forward(plan, srcs, dst)
    torch.cuda.synchronize()
    for t in dst:
        assert int(t.float().sum().item()) == tm.n_rows * 64


def test_misaligned_pointers_use_narrow_lanes():
    """Views that start 2 bytes into an allocation: only 2-byte alignment."""
    rng = np.random.default_rng(8)
    tm = wl.token_map_from_lens(rng, 1, 64, 24, [[10, 20]])
    src, dst = wl.Grid(dp=2), wl.Grid(tp=2, cp=2)
    plan = hp.hp_plan_create(src, dst, tm)
    prob = oracle.Problem(src, dst, tm)
    rows, drows, H = prob.src_rows(), prob.dst_rows(), 24

    def shifted(n_rows, seed):
        flat = wl.random_bf16((n_rows * H + 1,), seed).cuda()
        return flat[1:].view(n_rows, H)

    g_src = [shifted(r, 10 + i) for i, r in enumerate(rows)]
    g_dst = [shifted(drows, 20 + j) for j in range(prob.n_dst)]
    assert all(t.data_ptr() % 4 == 2 for t in g_src + g_dst)
    o_dst = [_to_host_bits(t).copy() for t in g_dst]
    hp.hp_forward(plan, g_src, g_dst)
    torch.cuda.synchronize()
    prob.forward([_to_host_bits(t) for t in g_src], o_dst)
    for j in range(prob.n_dst):
        assert np.array_equal(_to_host_bits(g_dst[j]), o_dst[j])
    g_sg = [shifted(r, 30 + i) for i, r in enumerate(rows)]
    hp.hp_backward(plan, g_dst, g_sg)
    torch.cuda.synchronize()
    o_sg = [np.zeros((r, H), np.uint16) for r in rows]
    prob.backward_bf16(o_dst, o_sg)
    for i in range(prob.n_src):
        assert np.array_equal(_to_host_bits(g_sg[i]), o_sg[i])


def test_empty_plan_and_null_empty_ranks():
    tm = wl.TokenMap(2, 16, 8, [], [], [])
    plan = hp.hp_plan_create(wl.Grid(dp=2), wl.Grid(tp=2), tm)
    d = [torch.ones((32, 8), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    hp.hp_forward(plan, [None, None], d)
    hp.hp_backward(plan, d, [None, None])
    torch.cuda.synchronize()
    assert bool((d[0] == 1).all())
    # one image, eight source ranks: seven are empty and may be passed as None
    tm = wl.TokenMap(1, 16, 8, [0], [3], [5])
    plan = hp.hp_plan_create(wl.Grid(dp=8), wl.Grid(), tm)
    rows = plan.src_rows()
    assert sorted(rows) == [0] * 7 + [5]
    srcs = [torch.full((r, 8), 2.0, dtype=torch.bfloat16, device="cuda") if r else None for r in rows]
    d = [torch.zeros((16, 8), dtype=torch.bfloat16, device="cuda")]
    hp.hp_forward(plan, srcs, d)
    torch.cuda.synchronize()
    assert d[0].float().sum().item() == 2.0 * 5 * 8 and bool((d[0][3:8] == 2).all())
    with pytest.raises(hp.HpError):
        hp.hp_forward(plan, [None] * 8, d)                  # the one non-empty rank is required


def test_caller_stream_and_determinism():
    """Runs on a caller-created stream; two runs give identical bits."""
    w = wl.scaled(wl.long_context(), 256)
    st = torch.cuda.Stream()
    check_case(w.src, w.dst, w.maps[0], seed=11, stream=st)
    plan = hp.hp_plan_create(w.src, w.dst, w.maps[0])
    g = [wl.random_bf16((plan.info.dst_rows_per_buf, 256), 50 + j, "cuda") for j in range(32)]
    outs = []
    for _ in range(2):
        sg = [torch.zeros((r, 256), dtype=torch.bfloat16, device="cuda") for r in plan.src_rows()]
        torch.cuda.synchronize()
        hp.hp_backward(plan, g, sg, st)
        st.synchronize()
        outs.append([t.view(torch.int16).clone() for t in sg])
    assert all(torch.equal(a, b) for a, b in zip(*outs))


def test_profile_records_kernel_durations():
    w = wl.scaled(wl.long_context(), 512)
    plan = hp.hp_plan_create(w.src, w.dst, w.maps[0])
    src = [wl.random_bf16((r, 512), 1 + i, "cuda") for i, r in enumerate(plan.src_rows())]
    dst = [torch.zeros((plan.info.dst_rows_per_buf, 512), dtype=torch.bfloat16, device="cuda") for _ in range(32)]
    sg = [torch.zeros_like(t) for t in src]
    hp.hp_profile_enable(3)
    try:
        hp.hp_forward(plan, src, dst)
        hp.hp_backward(plan, dst, sg)
        hp.hp_forward(plan, src, dst)
        hp.hp_backward(plan, dst, sg)            # beyond the 3 pairs: runs untimed
        got = hp.hp_profile_read(8)
        assert [k for k, _ in got] == [0, 1, 0]
        assert all(0.0 < ms < 50.0 for _, ms in got)
        assert hp.hp_profile_read(8) == []
    finally:
        hp.hp_profile_enable(0)
    torch.cuda.synchronize()
    for a, b in zip(sg, src):
        assert torch.equal(a.float(), 4.0 * b.float())    # four identical replicas summed: exact in bf16


def _guarded(rows, hidden, dtype, fill, guard=3):
    """A [rows, hidden] buffer cut out of a larger allocation whose `guard` rows
    before and after it hold a sentinel: (buffer view, whole allocation)."""
    whole = torch.full((rows + 2 * guard, hidden), fill, dtype=dtype, device="cuda")
    return whole[guard:guard + rows], whole


@pytest.mark.parametrize("case", ["random0", "random1", "random2", "random3", "long_context_h328", "sbh_short_rows",
                                  "seq_shard", "accumulate_f32"])
def test_guard_rows_around_every_buffer_stay_untouched(case):
    """Every buffer of a call sits between sentinel rows; forward, backward and
    the accumulating backward must leave all of them as found (an access past a
    buffer's end that lands in unrelated memory would go unnoticed by the
    whole-buffer comparisons)."""
    rng = np.random.default_rng(abs(hash(case)) % 1000)
    acc = case == "accumulate_f32"
    if case.startswith("random"):
        src, dst, tm = wl.random_layout_case(np.random.default_rng(900 + int(case[-1])))
    elif case == "sbh_short_rows":
        src, dst = wl.Grid(tp=2, dp=2), wl.Grid(tp=2, cp=2, dp=1, cp_split=wl.CP_ZIGZAG, row_order=wl.ROW_SBH)
        tm = wl.token_map_from_lens(rng, 4, 64, 24, [[5, 9], [17], [], [3, 3, 3]])
    else:
        w = wl.scaled(wl.long_context(), 328)                    # 656-byte rows: 16-byte lanes, ragged tiles
        src, dst, tm = w.src, w.dst, w.maps[0]
        if case == "seq_shard":
            dst = replace(dst, tp_mode=wl.TP_SEQ_SHARD)
    plan = hp.hp_plan_create(src, dst, tm)
    H, drows = tm.hidden, plan.info.dst_rows_per_buf
    S = 0x7FC5
    mk = lambda rows, dt, fill: _guarded(rows, H, dt, fill)
    bf = torch.bfloat16
    srcs = [mk(r, bf, 1.5) for r in plan.src_rows()]
    dsts = [mk(drows, bf, 2.5) for _ in range(plan.info.n_dst_bufs)]
    grads = [mk(drows, bf, 0.25) for _ in range(plan.info.n_dst_bufs)]
    sgs = [mk(r, torch.float32 if acc else bf, 7.0) for r in plan.src_rows()]
    for view, whole in srcs + dsts + grads + sgs:                # sentinels into the guard rows only
        raw = whole.view(torch.int16) if whole.dtype == bf else whole
        raw[:3] = S if whole.dtype == bf else -123.0
        raw[-3:] = S if whole.dtype == bf else -123.0
    torch.cuda.synchronize()
    hp.hp_forward(plan, [v for v, _ in srcs], [v for v, _ in dsts])
    if acc:
        hp.hp_backward_accumulate(plan, [v for v, _ in grads], [v for v, _ in sgs])
    else:
        hp.hp_backward(plan, [v for v, _ in grads], [v for v, _ in sgs])
    hp.hp_forward_static(plan, [v for v, _ in srcs], [v for v, _ in dsts])
    zeroed = [mk(drows, bf, 4.5) for _ in range(plan.info.n_dst_bufs)]
    for view, whole in zeroed:
        whole.view(torch.int16)[:3] = S
        whole.view(torch.int16)[-3:] = S
    torch.cuda.synchronize()
    hp.hp_zero_image_rows(plan, [v for v, _ in zeroed])
    torch.cuda.synchronize()
    assert sum(int((v == 0).all(dim=1).sum()) for v, _ in zeroed) == plan.info.dst_copies * tm.n_rows
    for name, group in (("source", srcs), ("destination", dsts), ("gradient", grads), ("source gradient", sgs),
                        ("zeroed", zeroed)):
        for i, (view, whole) in enumerate(group):
            g = torch.cat([whole[:3], whole[-3:]])
            if whole.dtype == bf:
                assert bool((g.view(torch.int16) == torch.tensor(S, dtype=torch.int16)).all()), (name, i)
            else:
                assert bool((g == -123.0).all()), (name, i)
    # and the calls did their work: image rows moved (1.5), source gradients written
    n_img = sum(int((v == 1.5).all(dim=1).sum()) for v, _ in dsts)
    assert n_img == plan.info.dst_copies * tm.n_rows
    want = (0.25 * plan.info.dst_copies) + (7.0 if acc else 0.0)
    for (v, _), r in zip(sgs, plan.src_rows()):
        assert r == 0 or bool((v == want).all())
    plan.close()


@pytest.mark.parametrize("seed", range(10))
def test_zero_image_rows_random_layouts(seed):
    """hp_zero_image_rows against the oracle: bf16 and binary32 buffers, both TP
    modes and row orders, whole buffers compared."""
    rng = np.random.default_rng(1200 + seed)
    src, dst, tm = wl.random_layout_case(rng)
    if seed % 3 == 2 and (tm.seq // dst.cp) % dst.tp == 0:
        dst = replace(dst, tp_mode=wl.TP_SEQ_SHARD)
    for dtype, tdt, ndt in ((wl.DT_BF16, torch.bfloat16, np.uint16), (wl.DT_F32, torch.float32, np.float32)):
        tmd = replace(tm, dtype=dtype)
        plan = hp.hp_plan_create(src, dst, tmd)
        prob = oracle.Problem(src, dst, tmd)
        bufs = [(torch.randn((prob.dst_rows(), tm.hidden), generator=torch.Generator().manual_seed(seed * 50 + j)) + 3.0)
                .to(tdt).cuda() for j in range(prob.n_dst)]
        host = lambda t: (t.cpu().contiguous().view(torch.int16).numpy().view(np.uint16) if ndt is np.uint16
                          else t.cpu().numpy()).copy()
        want = [host(t) for t in bufs]
        prob.zero_image_rows(want)
        torch.cuda.synchronize()
        hp.hp_zero_image_rows(plan, bufs)
        torch.cuda.synchronize()
        for j in range(prob.n_dst):
            assert np.array_equal(host(bufs[j]), want[j]), (seed, j)
        plan.close()


def test_zero_image_rows_long_context_spans_and_strided_rows():
    for hidden, order in ((328, wl.ROW_BSH), (7, wl.ROW_BSH), (2048, wl.ROW_BSH)):
        w = wl.scaled(wl.long_context(), hidden)
        tm = w.maps[0]
        plan = hp.hp_plan_create(w.src, w.dst, tm)
        prob = oracle.Problem(w.src, w.dst, tm)
        bufs = [wl.random_bf16((prob.dst_rows(), hidden), 700 + j, "cuda") for j in range(prob.n_dst)]
        want = [_to_host_bits(t).copy() for t in bufs]
        prob.zero_image_rows(want)
        torch.cuda.synchronize()
        hp.hp_zero_image_rows(plan, bufs)
        torch.cuda.synchronize()
        assert all(np.array_equal(_to_host_bits(t), w_) for t, w_ in zip(bufs, want))
        plan.close()
    w = wl.scaled(wl.colocated4(), 24)                           # four samples per rank, [S,B,H]: row-strided segments
    dst = replace(w.dst, row_order=wl.ROW_SBH)
    plan = hp.hp_plan_create(w.src, dst, w.maps[0])
    prob = oracle.Problem(w.src, dst, w.maps[0])
    bufs = [wl.random_bf16((prob.dst_rows(), 24), 800 + j, "cuda") for j in range(prob.n_dst)]
    want = [_to_host_bits(t).copy() for t in bufs]
    prob.zero_image_rows(want)
    torch.cuda.synchronize()
    hp.hp_zero_image_rows(plan, bufs)
    torch.cuda.synchronize()
    assert all(np.array_equal(_to_host_bits(t), w_) for t, w_ in zip(bufs, want))
    plan.close()


@pytest.mark.parametrize("seed", range(6))
def test_autograd_wrapper_against_torch_autograd_of_the_definition(seed):
    """boundary_transform (hp_forward / hp_backward / hp_zero_image_rows under
    torch.autograd) against CPU torch autograd of the definition written with
    index_copy, binary32 payloads with small integers (every sum exact, so the
    result does not depend on an accumulation order)."""
    rng = np.random.default_rng(1300 + seed)
    src, dst, tm = wl.random_layout_case(rng)
    tm = replace(tm, dtype=wl.DT_F32)
    plan = hp.hp_plan_create(src, dst, tm)
    prob = oracle.Problem(src, dst, tm)
    H, rows, drows = tm.hidden, prob.src_rows(), prob.dst_rows()
    ints = lambda shape: torch.from_numpy(rng.integers(-6, 7, size=shape).astype(np.float32))
    x_cpu = [ints((r, H)) for r in rows]
    t_cpu = [ints((drows, H)) for _ in range(prob.n_dst)]
    w_cpu = [ints((drows, H)) for _ in range(prob.n_dst)]           # weights of a scalar loss
    # --- reference: the definition under CPU autograd (forward reads the leader copy tp = 0 only) ---
    xr = [t.clone().requires_grad_(True) for t in x_cpu]
    tr = [t.clone().requires_grad_(True) for t in t_cpu]
    loss = 0.0
    for j in range(prob.n_dst):
        sb, sr = prob.forward_map(j)
        img = np.nonzero(sb >= 0)[0]
        out = tr[j]
        for b in sorted(set(sb[img].tolist())):
            sel = img[sb[img] == b]
            out = out.index_copy(0, torch.from_numpy(sel), xr[b][torch.from_numpy(sr[sel])])
        loss = loss + (out * w_cpu[j]).sum()
    loss.backward()
    # --- the library under autograd ---
    xg = [t.clone().cuda().requires_grad_(True) for t in x_cpu]
    tg = [t.clone().cuda().requires_grad_(True) for t in t_cpu]
    outs = hp.boundary_transform(plan, xg, [t.clone() for t in tg])    # clones: leaves cannot be modified in place
    gl = sum((o * w.cuda()).sum() for o, w in zip(outs, w_cpu))
    gl.backward()
    torch.cuda.synchronize()
    for j in range(prob.n_dst):
        assert torch.equal(tg[j].grad.cpu(), tr[j].grad), ("text gradient", j)
    for i in range(prob.n_src):
        leader = i - i % src.tp
        want = xr[leader].grad if xr[leader].grad is not None else torch.zeros_like(x_cpu[i])
        # every TP copy of a source rank receives the gradient of the rank's rows
        assert torch.equal(xg[i].grad.cpu(), want), ("source gradient", i)
    plan.close()


# ---- full sizes, in the launch configuration the benchmark times --------------

def test_full_colocated4():
    w = wl.colocated4()
    info = check_case(w.src, w.dst, w.maps[0], seed=2, gen_device="cuda")
    assert info.boundary_bytes == 256 << 20


def test_full_colocated4_dense_reading():
    """Config 2 read with a fused length of 8192: images tile the sequences."""
    w = wl.colocated4_dense()
    info = check_case(w.src, w.dst, w.maps[0], seed=22, gen_device="cuda")
    assert info.boundary_bytes == 256 << 20 and info.n_rows == 4 * 8192


def test_full_long_context():
    w = wl.long_context()
    info = check_case(w.src, w.dst, w.maps[0], seed=3, gen_device="cuda")
    assert info.dst_copies == 4 and info.row_bytes == 10240


def test_full_long_context_in_tuned_launch_shapes():
    """The benchmark's configuration: hp_plan_tune first, then the full-size
    comparison on a plan that starts from the remembered shapes."""
    w = wl.long_context()
    tm = w.maps[0]
    plan = hp.hp_plan_create(w.src, w.dst, tm)
    rows, drows, H = plan.src_rows(), plan.info.dst_rows_per_buf, tm.hidden
    src = [wl.random_bf16((r, H), 5 + i, "cuda") for i, r in enumerate(rows)]
    dst = [torch.empty((drows, H), dtype=torch.bfloat16, device="cuda") for _ in range(32)]
    grad = [wl.random_bf16((drows, H), 90 + j, "cuda") for j in range(32)]
    sg = [torch.empty((r, H), dtype=torch.bfloat16, device="cuda") for r in rows]
    hp.hp_plan_tune(plan, src, dst, grad, sg, torch.cuda.current_stream())
    tuned = (plan.get_launch(0), plan.get_launch(1))
    plan.close()
    del src, dst, grad, sg
    check_case(w.src, w.dst, tm, seed=33, gen_device="cuda", expect_launch=tuned)


def test_full_non_colocated_microbatches():
    w = wl.non_colocated()
    for i in (0, 7, 15):
        check_case(w.src, w.dst, w.maps[i], seed=40 + i, gen_device="cuda")


def test_full_large_scale():
    w = wl.large_scale()
    info = check_case(w.src, w.dst, w.maps[0], seed=5, gen_device="cuda")
    assert (info.src_copies, info.dst_copies) == (2, 8)


@pytest.mark.parametrize("name,hidden", [("non_colocated", 256), ("large_scale", 256), ("long_context", 320)])
def test_contiguous_cp_split_on_the_named_grids(name, hidden):
    """The paper gives no CP split rule; the load-balanced one is primary and the
    contiguous one is checked on the same grids and token maps (config 4:
    microbatches 0, 7 and 15 and the batched plan; configs 5 and 3: the whole
    map), at a reduced hidden size."""
    w = wl.scaled(wl.CONFIGS[name](), hidden)
    dst = replace(w.dst, cp_split=wl.CP_CONTIGUOUS)
    for i in ([0, 7, 15] if len(w.maps) > 1 else [0]):
        info = check_case(w.src, dst, w.maps[i], seed=60 + i, gen_device="cuda")
        assert info.n_rows == w.maps[i].n_rows
    if len(w.maps) > 1:
        _batched_case(replace(w, dst=dst), hidden, seed=6)
    check_case_extended(w.src, dst, w.maps[0], seed=61)


# ---- batched plans and the tuner ------------------------------------------------

def _batched_case(w, hidden, seed):
    """One batched plan over all microbatches vs the oracle run per microbatch."""
    maps = [replace(m, hidden=hidden) for m in w.maps]
    plan = hp.hp_plan_create_batched(w.src, w.dst, maps)
    n_src, n_dst = w.src.n_ranks, w.dst.n_ranks
    rows, drows = plan.src_rows(), plan.info.dst_rows_per_buf
    src = [wl.random_bf16((r, hidden), seed * 977 + i, "cuda") for i, r in enumerate(rows)]
    dst = [wl.random_bf16((drows, hidden), seed * 977 + 400 + j, "cuda") for j in range(plan.info.n_dst_bufs)]
    grad = [wl.random_bf16((drows, hidden), seed * 977 + 800 + j, "cuda") for j in range(plan.info.n_dst_bufs)]
    pre = [_to_host_bits(t).copy() for t in dst]
    sg = [torch.full((r, hidden), 7.0, dtype=torch.bfloat16, device="cuda") for r in rows]
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    hp.hp_forward(plan, src, dst, st)
    hp.hp_backward(plan, grad, sg, st)
    st.synchronize()
    for mi, tm in enumerate(maps):
        prob = oracle.Problem(w.src, w.dst, tm)
        o_dst = pre[mi * n_dst:(mi + 1) * n_dst]
        prob.forward([_to_host_bits(t) for t in src[mi * n_src:(mi + 1) * n_src]], o_dst)
        for j in range(n_dst):
            assert np.array_equal(_to_host_bits(dst[mi * n_dst + j]), o_dst[j]), (mi, j)
        o_sg = [np.zeros((r, hidden), np.uint16) for r in prob.src_rows()]
        prob.backward_bf16([_to_host_bits(t) for t in grad[mi * n_dst:(mi + 1) * n_dst]], o_sg)
        for i in range(n_src):
            assert np.array_equal(_to_host_bits(sg[mi * n_src + i]), o_sg[i]), (mi, i)
    return plan


def test_batched_plan_small():
    _batched_case(wl.non_colocated(n_microbatches=5), 72, seed=1)


def test_batched_plan_full_non_colocated():
    """All 16 microbatches of config 4 at full size in one launch per direction."""
    plan = _batched_case(wl.non_colocated(), 8192, seed=2)
    assert plan.info.n_maps == 16 and plan.info.n_src_bufs == 64 and plan.info.n_dst_bufs == 64


def test_tune_keeps_results_exact_and_picks_a_valid_shape():
    H = 2816                                   # forward moves 1.13 GB: above the size the tuner searches from
    w = wl.scaled(wl.long_context(), H)
    tm = w.maps[0]
    plan = hp.hp_plan_create(w.src, w.dst, tm)
    prob = oracle.Problem(w.src, w.dst, tm)
    rows, drows = plan.src_rows(), plan.info.dst_rows_per_buf
    src = [wl.random_bf16((r, H), 5 + i, "cuda") for i, r in enumerate(rows)]
    dst = [wl.random_bf16((drows, H), 50 + j, "cuda") for j in range(32)]
    grad = [wl.random_bf16((drows, H), 90 + j, "cuda") for j in range(32)]
    pre = [_to_host_bits(t).copy() for t in dst]
    sg = [torch.zeros((r, H), dtype=torch.bfloat16, device="cuda") for r in rows]
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    hp.hp_plan_tune(plan, src, dst, grad, sg, st)
    for d in (0, 1):
        L = plan.get_launch(d)
        assert L["tile_bytes"] in (1024, 2048, 4096, 8192) and L["block_threads"] in (64, 128, 256)
        assert 0 <= L["waves_per_cu"] <= 32
    # the buffers hold what one forward / backward would have produced
    prob.forward([_to_host_bits(t) for t in src], pre)
    o_sg = [np.zeros((r, H), np.uint16) for r in rows]
    prob.backward_bf16([_to_host_bits(t) for t in grad], o_sg)
    for j in range(32):
        assert np.array_equal(_to_host_bits(dst[j]), pre[j])
    for i in range(8):
        assert np.array_equal(_to_host_bits(sg[i]), o_sg[i])
    # and the tuned plan still computes the same thing
    sg2 = [torch.zeros_like(t) for t in sg]
    hp.hp_backward(plan, grad, sg2, st)
    st.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(sg, sg2))
    hp.hp_plan_tune(plan, src, dst, None, None, st)          # one direction only
    # a later plan of the same problem class starts from the tuned shapes
    tuned = (plan.get_launch(0), plan.get_launch(1))
    other = hp.hp_plan_create(w.src, w.dst, wl.scaled(wl.long_context(n_images=5), H).maps[0])
    assert (other.get_launch(0), other.get_launch(1)) == tuned
    hp.hp_forget_tuned_shapes()
    fresh = hp.hp_plan_create(w.src, w.dst, tm)
    untuned = hp.hp_plan_create_host(w.src, w.dst, tm)
    assert [fresh.get_launch(d) for d in (0, 1, 2)] == [untuned.get_launch(d) for d in (0, 1, 2)]
    assert fresh.get_launch(0) == dict(tile_bytes=2048, block_threads=64, waves_per_cu=12, nontemporal=2)


def test_tune_accumulate_picks_a_valid_shape_and_keeps_the_sum_exact():
    H = 2048                                   # 1.3 GB per accumulating launch: searched
    w = wl.scaled(wl.long_context(), H)
    tm = w.maps[0]
    plan = hp.hp_plan_create(w.src, w.dst, tm)
    prob = oracle.Problem(w.src, w.dst, tm)
    rows, drows = plan.src_rows(), plan.info.dst_rows_per_buf
    grad = [wl.random_bf16((drows, H), 190 + j, "cuda") for j in range(32)]
    scratch = [torch.zeros((r, H), dtype=torch.float32, device="cuda") for r in rows]
    plan.tune_accumulate(grad, scratch, torch.cuda.current_stream())
    L = plan.get_launch(2)
    assert L["tile_bytes"] in (1024, 2048, 4096, 8192) and L["block_threads"] in (64, 128, 256)
    other = hp.hp_plan_create(w.src, w.dst, wl.scaled(wl.long_context(n_images=4), H).maps[0])
    assert other.get_launch(2) == L                     # remembered for the problem class
    acc = [torch.zeros_like(t) for t in scratch]
    hp.hp_backward_accumulate(plan, grad, acc)
    torch.cuda.synchronize()
    want = [np.zeros((r, H), np.float32) for r in rows]
    prob.backward_accumulate([_to_host_bits(t) for t in grad], want)
    for a, b in zip(acc, want):
        assert np.array_equal(a.cpu().numpy().view(np.uint32), b.view(np.uint32))
    # a small plan keeps its shape
    small = hp.hp_plan_create(w.src, w.dst, wl.scaled(wl.long_context(n_images=4), 64).maps[0])
    before = small.get_launch(2)
    g2 = [wl.random_bf16((drows, 64), 7 + j, "cuda") for j in range(32)]
    small.tune_accumulate(g2, [torch.zeros((r, 64), dtype=torch.float32, device="cuda") for r in small.src_rows()])
    assert small.get_launch(2) == before


def test_tune_leaves_small_plans_alone():
    """Less than 1 GiB per forward launch: no search (it would be timed out of
    the memory-side cache); the buffers still end up as after one call."""
    w = wl.scaled(wl.long_context(n_images=6), 256)
    tm = w.maps[0]
    plan = hp.hp_plan_create(w.src, w.dst, tm)
    before = [plan.get_launch(d) for d in (0, 1, 2)]
    prob = oracle.Problem(w.src, w.dst, tm)
    src, pre, grads = make_inputs(prob, 12, "cuda")
    dst = [t.clone() for t in pre]
    sg = [torch.zeros_like(t) for t in src]
    hp.hp_plan_tune(plan, src, dst, grads, sg, torch.cuda.current_stream())
    assert [plan.get_launch(d) for d in (0, 1, 2)] == before
    want = [_to_host_bits(t).copy() for t in pre]
    prob.forward([_to_host_bits(t) for t in src], want)
    o_sg = [np.zeros((r, 256), np.uint16) for r in prob.src_rows()]
    prob.backward_bf16([_to_host_bits(t) for t in grads], o_sg)
    assert all(np.array_equal(_to_host_bits(a), b) for a, b in zip(dst, want))
    assert all(np.array_equal(_to_host_bits(a), b) for a, b in zip(sg, o_sg))
    other = hp.hp_plan_create(w.src, w.dst, tm)          # nothing was remembered for this problem class
    assert [other.get_launch(d) for d in (0, 1, 2)] == before


def test_stream_probe_reports_a_rate():
    gbps, shape = hp.hp_probe_stream(1, 4, 8 << 20)
    assert gbps > 50.0 and shape["tile_bytes"] in (1024, 2048, 4096, 8192)
    fixed = dict(tile_bytes=4096, block_threads=256, waves_per_cu=16, nontemporal=2)
    gbps2, shape2 = hp.hp_probe_stream(4, 1, 8 << 20, fixed)
    assert gbps2 > 50.0 and shape2 == fixed
    with pytest.raises(hp.HpError):
        hp.hp_probe_stream(9, 1, 8 << 20)
    # other tile schedules of the probe (ragged sizes: the last tile and the last XCD share are partial)
    for sched in ("oneshot", "xcd_chunked", "persistent", "persistent_xcd", "phased"):
        for nbytes in (8 << 20, (8 << 20) + 4096 + 16, 65536):
            assert hp.hp_probe_stream_ex(1, 4, nbytes, fixed, sched) > 1.0
            if sched != "phased":                                # phased: one read stream at most, one write at least
                assert hp.hp_probe_stream_ex(2, 0, nbytes, dict(fixed, block_threads=256, tile_bytes=8192), sched) > 1.0
    with pytest.raises(hp.HpError):
        hp.hp_probe_stream_ex(0, 0, 8 << 20, fixed, 0)
    with pytest.raises(hp.HpError):
        hp.hp_probe_stream_ex(1, 1, 8 << 20, fixed, 7)
    with pytest.raises(hp.HpError):
        hp.hp_probe_stream_ex(2, 1, 8 << 20, fixed, "phased")
    for tile, block in ((65536, 256), (65536, 512), (65536, 1024), (16384, 256)):      # 16, 8, 4, 4 chunks per lane
        deep = dict(tile_bytes=tile, block_threads=block, waves_per_cu=16, nontemporal=2)
        assert hp.hp_probe_stream_ex(1, 4, (8 << 20) + 4096 + 16, deep, "phased") > 1.0


# ---- binary32 payloads and the accumulating backward ---------------------------

@pytest.mark.parametrize("seed", range(12))
def test_f32_and_accumulate_random_layouts(seed):
    from parity import check_case_extended
    rng = np.random.default_rng(700 + seed)
    src, dst, tm = wl.random_layout_case(rng)
    check_case_extended(src, dst, replace(tm, dtype=wl.DT_F32), seed=seed)
    check_case_extended(src, dst, tm, seed=seed)                     # bf16 gradients into f32 accumulators


@pytest.mark.parametrize("hidden,dtype", [(7, 0), (7, 1), (12, 0), (320, 0), (320, 1), (1022, 0), (2560, 1)])
def test_f32_and_accumulate_long_context_spans(hidden, dtype):
    from parity import check_case_extended
    w = wl.long_context(n_images=9)
    check_case_extended(w.src, w.dst, replace(w.maps[0], hidden=hidden, dtype=dtype), seed=hidden)


@pytest.mark.parametrize("tile,block,waves,nt", [(1024, 64, 16, 3), (2048, 64, 14, 3), (1024, 128, 0, 0),
                                                 (8192, 256, 8, 1), (65536, 1024, 32, 2), (2048, 256, 4, 3)])
def test_accumulate_launch_shapes(tile, block, waves, nt):
    """hp_backward_accumulate in launch shapes its tuner may pick (small tiles
    included), bf16 and binary32 gradients, ragged tile ends."""
    from parity import check_case_extended
    w = wl.scaled(wl.long_context(n_images=9), 264)
    shape = dict(tile_bytes=tile, block_threads=block, waves_per_cu=waves, nontemporal=nt)
    check_case_extended(w.src, w.dst, w.maps[0], seed=tile % 89, acc_launch=shape)
    check_case_extended(w.src, w.dst, replace(w.maps[0], dtype=wl.DT_F32), seed=tile % 83, acc_launch=shape)
    w5 = wl.scaled(wl.large_scale(), 72)                         # TP_dst 8, two source copies
    check_case_extended(w5.src, w5.dst, w5.maps[0], seed=block, acc_launch=shape)


def test_accumulate_large_scale_replicas():
    """TP_dst = 8, TP_src = 2 (both source copies accumulate), hidden 96."""
    from parity import check_case_extended
    w = wl.scaled(wl.large_scale(), 96)
    check_case_extended(w.src, w.dst, w.maps[0], seed=9)
    check_case_extended(w.src, w.dst, replace(w.maps[0], dtype=wl.DT_F32), seed=10)


# ---- batch-shard cases of the figures and joins of several edges ----------------

@pytest.mark.parametrize("dp_src,dp_dst", [(4, 2), (2, 4), (4, 4), (8, 1), (1, 4)])
def test_fan_in_fan_out_equal_dp(dp_src, dp_dst):
    """Fan-in (DP_src > DP_dst), fan-out (DP_src < DP_dst) and equal DP with
    different TP widths on the two sides, several samples per rank."""
    rng = np.random.default_rng(dp_src * 10 + dp_dst)
    batch = 8
    tm = wl.token_map_from_lens(rng, batch, 48, 40, [[int(x) for x in rng.integers(1, 9, size=3)] for _ in range(batch)])
    check_case(wl.Grid(tp=2, dp=dp_src), wl.Grid(tp=3, cp=2, dp=dp_dst, cp_split=wl.CP_ZIGZAG), tm, seed=dp_src)
    check_case(wl.Grid(tp=1, dp=dp_src), wl.Grid(tp=2, cp=1, dp=dp_dst, row_order=wl.ROW_SBH), tm, seed=dp_dst)


def test_two_edges_join_in_one_sequence():
    """Two encoders (say images and audio) feed disjoint spans of the same LLM
    sequence through two plans, one per edge; backward routes each gradient
    through the plan of the edge that produced the activation."""
    rng = np.random.default_rng(77)
    B, S, H = 2, 256, 64
    dst = wl.Grid(tp=2, cp=2, dp=1, cp_split=wl.CP_ZIGZAG)
    # interleave the two modalities' spans: even slots of 16 tokens to edge A, odd slots to edge B
    slots = [(b, s) for b in range(B) for s in range(0, S, 16) if rng.random() < 0.6]
    A = [x for i, x in enumerate(slots) if i % 2 == 0]
    Bm = [x for i, x in enumerate(slots) if i % 2 == 1]
    mk = lambda sp, ln: wl.TokenMap(B, S, H, [b for b, _ in sp], [s for _, s in sp], [ln] * len(sp))
    tm_a, tm_b = mk(A, 16), mk(Bm, 11)
    src_a, src_b = wl.Grid(tp=1, dp=4), wl.Grid(tp=2, dp=2, rank_offset=4)
    pa, pb = hp.hp_plan_create(src_a, dst, tm_a), hp.hp_plan_create(src_b, dst, tm_b)
    oa, ob = oracle.Problem(src_a, dst, tm_a), oracle.Problem(src_b, dst, tm_b)
    xa = [wl.random_bf16((r, H), 1 + i) for i, r in enumerate(pa.src_rows())]
    xb = [wl.random_bf16((r, H), 20 + i) for i, r in enumerate(pb.src_rows())]
    pre = [wl.random_bf16((pa.info.dst_rows_per_buf, H), 40 + j) for j in range(4)]
    g_dst = [t.cuda() for t in pre]
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    hp.hp_forward(pa, [t.cuda() for t in xa], g_dst, st)
    hp.hp_forward(pb, [t.cuda() for t in xb], g_dst, st)
    grads = [wl.random_bf16((pa.info.dst_rows_per_buf, H), 60 + j, "cuda") for j in range(4)]
    ga = [torch.zeros((r, H), dtype=torch.bfloat16, device="cuda") for r in pa.src_rows()]
    gb = [torch.zeros((r, H), dtype=torch.bfloat16, device="cuda") for r in pb.src_rows()]
    hp.hp_backward(pa, grads, ga, st)
    hp.hp_backward(pb, grads, gb, st)
    st.synchronize()
    o_dst = [_to_host_bits(t).copy() for t in pre]
    oa.forward([_to_host_bits(t) for t in xa], o_dst)
    ob.forward([_to_host_bits(t) for t in xb], o_dst)
    for j in range(4):
        assert np.array_equal(_to_host_bits(g_dst[j]), o_dst[j])
    hg = [_to_host_bits(t) for t in grads]
    for prob, got in ((oa, ga), (ob, gb)):
        want = [np.zeros((r, H), np.uint16) for r in prob.src_rows()]
        prob.backward_bf16(hg, want)
        for a, b in zip(got, want):
            assert np.array_equal(_to_host_bits(a), b)


def test_calls_can_be_captured_in_a_hip_graph():
    """hp_forward + hp_backward recorded into a graph by a capturing caller and
    replayed several times, with eager work and synchronisations between the
    replays; every replay must reproduce the eager result bit for bit."""
    w = wl.scaled(wl.long_context(), 384)
    tm = w.maps[0]
    plan = hp.hp_plan_create(w.src, w.dst, tm)
    rows, drows = plan.src_rows(), plan.info.dst_rows_per_buf
    src = [wl.random_bf16((r, 384), 3 + i, "cuda") for i, r in enumerate(rows)]
    pre = [wl.random_bf16((drows, 384), 40 + j, "cuda") for j in range(32)]
    dst = [t.clone() for t in pre]
    sg = [torch.zeros_like(t) for t in src]
    # eager reference
    hp.hp_forward(plan, src, dst)
    hp.hp_backward(plan, dst, sg)
    torch.cuda.synchronize()
    want_dst = [t.clone() for t in dst]
    want_sg = [t.clone() for t in sg]
    st = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(g, stream=st):
        hp.hp_forward(plan, src, dst, torch.cuda.current_stream())
        hp.hp_backward(plan, dst, sg, torch.cuda.current_stream())
    for rep in range(3):
        for t, p0 in zip(dst, pre):
            t.copy_(p0)                        # eager work between replays: restore the prefill,
        for t in sg:
            t.fill_(float(rep))                # scribble on the outputs
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert all(torch.equal(a.view(torch.int16), b.view(torch.int16)) for a, b in zip(dst, want_dst)), rep
        assert all(torch.equal(a.view(torch.int16), b.view(torch.int16)) for a, b in zip(sg, want_sg)), rep


def test_plans_rebuilt_every_step_reuse_device_blocks():
    """Token maps change every step: create, use and destroy 40 plans in a row
    (device table blocks are recycled) and check each result."""
    rng = np.random.default_rng(99)
    src, dst = wl.Grid(dp=4), wl.Grid(tp=2, cp=2, cp_split=wl.CP_ZIGZAG)
    H = 128
    for step in range(40):
        lens = [int(x) for x in rng.integers(1, 40, size=int(rng.integers(1, 9)))]
        tm = wl.token_map_from_lens(rng, 1, 512, H, [lens])
        plan = hp.hp_plan_create(src, dst, tm)
        prob = oracle.Problem(src, dst, tm)
        xs = [wl.random_bf16((r, H), step * 10 + i) for i, r in enumerate(plan.src_rows())]
        pre = [wl.random_bf16((plan.info.dst_rows_per_buf, H), step * 10 + 5 + j) for j in range(4)]
        g_dst = [t.cuda() for t in pre]
        hp.hp_forward(plan, [t.cuda() if t.numel() else None for t in xs], g_dst)
        torch.cuda.synchronize()
        plan.close()
        want = [_to_host_bits(t).copy() for t in pre]
        prob.forward([_to_host_bits(t) for t in xs], want)
        for j in range(4):
            assert np.array_equal(_to_host_bits(g_dst[j]), want[j]), (step, j)
    hp.hp_release_cached_memory()


def test_batched_plan_at_the_buffer_limit():
    """56 microbatches x (4 source + 4 destination) buffers = 448 pointers, the
    most one plan accepts; one more microbatch is refused."""
    w = wl.non_colocated(n_microbatches=57)
    big = replace(w, maps=w.maps[:56])
    plan = _batched_case(big, 64, seed=3)
    assert plan.info.n_src_bufs + plan.info.n_dst_bufs == 448
    with pytest.raises(hp.HpError):
        hp.hp_plan_create_batched(w.src, w.dst, [replace(m, hidden=64) for m in w.maps])


def test_sequence_sharded_destination_long_context_spans():
    """Config-3 spans with TP ranks holding sequence shards: pieces of 4096
    positions, so spans are cut at zigzag chunk borders and at shard borders."""
    w = wl.long_context()
    tm = replace(w.maps[0], hidden=192)
    info = check_case(w.src, replace(w.dst, tp_mode=wl.TP_SEQ_SHARD), tm, seed=12)
    assert info.dst_copies == 1 and info.dst_rows_per_buf == 4096
    check_case(w.src, replace(w.dst, tp_mode=wl.TP_SEQ_SHARD, cp_split=wl.CP_CONTIGUOUS), tm, seed=13)


def test_plan_destroyed_while_its_calls_are_still_queued():
    """hp_plan_destroy right after the calls were enqueued, followed by a new
    plan that takes over the recycled device block: the queued calls must still
    run on their own tables.  Both token maps have the same span lengths and the
    same segment and tile structure (spans well inside the sequence chunks, the
    second map shifted by 37 rows), and all buffers have the same sizes."""
    H, S = 2048, 65536
    src, dst = wl.Grid(dp=2), wl.Grid(tp=2, cp=2, cp_split=wl.CP_ZIGZAG)
    starts = np.array([1000, 20000, 36000, 50000])
    tm_a = wl.TokenMap(1, S, H, [0] * 4, starts, [6000] * 4)
    tm_b = wl.TokenMap(1, S, H, [0] * 4, starts + 37, [6000] * 4)
    prob_a, prob_b = oracle.Problem(src, dst, tm_a), oracle.Problem(src, dst, tm_b)
    assert prob_a.src_rows() == prob_b.src_rows()
    hp.hp_release_cached_memory()                         # so that plan b can only get plan a's block
    plan_a = hp.hp_plan_create(src, dst, tm_a)
    q = hp.hp_plan_create_host(src, dst, tm_b)
    assert plan_a.info.n_segments == q.info.n_segments and plan_a.info.n_tiles == q.info.n_tiles
    q.close()
    srcs, pre, _ = make_inputs(prob_a, 77, "cuda")
    dst_a = [t.clone() for t in pre]
    dst_b = [t.clone() for t in pre]
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    ps, pd = plan_a.pointer_arrays(srcs, dst_a)
    for _ in range(40):                                   # ~2 ms of queued work
        plan_a.forward_raw(ps, pd, st)
    plan_a.close()                                        # no synchronisation before this
    plan_b = hp.hp_plan_create(src, dst, tm_b)            # reuses the block once the queue has drained
    hp.hp_forward(plan_b, srcs, dst_b, st)
    torch.cuda.synchronize()
    h_src = [_to_host_bits(t) for t in srcs]
    for prob, got in ((prob_a, dst_a), (prob_b, dst_b)):
        want = [_to_host_bits(t).copy() for t in pre]
        prob.forward(h_src, want)
        for j in range(prob.n_dst):
            assert np.array_equal(_to_host_bits(got[j]), want[j]), j
    plan_b.close()


@pytest.mark.parametrize("seed", range(6))
def test_joined_plan_one_launch_for_all_edges(seed):
    """Two or three encoders with different grids (different TP widths, so the
    backward writes a different number of copies per edge) join one sequence,
    two microbatches: one hp_forward and one hp_backward launch for everything,
    checked against the oracle applied edge by edge and microbatch by
    microbatch.  Also the accumulating backward."""
    rng = np.random.default_rng(900 + seed)
    n_edges, n_maps = 2 + seed % 2, 2
    B, S, H = 2, 512, (64, 40, 7)[seed % 3]
    dst = wl.Grid(tp=(2, 3, 4)[seed % 3], cp=2, dp=1 + seed % 2, cp_split=wl.CP_ZIGZAG if seed % 2 else wl.CP_CONTIGUOUS,
                  tp_mode=wl.TP_SEQ_SHARD if seed in (3, 5) else wl.TP_REPLICATE,
                  row_order=wl.ROW_SBH if seed == 2 else wl.ROW_BSH)
    srcs = [wl.Grid(tp=1 + (e + seed) % 2, dp=int(rng.choice([1, 2, 3, 4])), rank_offset=16 * e) for e in range(n_edges)]
    maps = [[None] * n_maps for _ in range(n_edges)]
    for m in range(n_maps):
        lens = [[int(x) for x in rng.integers(1, 60, size=int(rng.integers(1, 6)))] for _ in range(B)]
        tm = wl.token_map_from_lens(rng, B, S, H, lens)
        for e, part in enumerate(wl.split_edges(rng, tm, n_edges)):
            maps[e][m] = part
    plan = hp.hp_plan_create_joined(srcs, dst, maps)
    n_dst = dst.tp * dst.cp * dst.dp
    drows = plan.info.dst_rows_per_buf
    rows = plan.src_rows()
    x = [wl.random_bf16((r, H), 1000 * seed + i) for i, r in enumerate(rows)]
    pre = [wl.random_bf16((drows, H), 1000 * seed + 300 + j) for j in range(n_dst * n_maps)]
    grads = [wl.random_bf16((drows, H), 1000 * seed + 600 + j) for j in range(n_dst * n_maps)]
    acc0 = [torch.randn((r, H), generator=torch.Generator().manual_seed(seed * 31 + i)) for i, r in enumerate(rows)]
    g_dst = [t.cuda() for t in pre]
    g_sg = [torch.full((r, H), float("nan"), dtype=torch.bfloat16, device="cuda") for r in rows]
    g_acc = [t.cuda() for t in acc0]
    g_grads = [t.cuda() for t in grads]
    hp.hp_forward(plan, [t.cuda() for t in x], g_dst)
    hp.hp_backward(plan, g_grads, g_sg)
    hp.hp_backward_accumulate(plan, g_grads, g_acc)
    torch.cuda.synchronize()
    # oracle, one (edge, microbatch) at a time
    o_dst = [_to_host_bits(t).copy() for t in pre]
    base = 0
    for e in range(n_edges):
        per_map = srcs[e].tp * srcs[e].dp
        for m in range(n_maps):
            prob = oracle.Problem(srcs[e], dst, maps[e][m])
            sl = slice(base + m * per_map, base + (m + 1) * per_map)
            dl = slice(m * n_dst, (m + 1) * n_dst)
            assert rows[sl] == prob.src_rows()
            prob.forward([_to_host_bits(t) for t in x[sl]], o_dst[dl])
            hg = [_to_host_bits(t) for t in grads[dl]]
            want = [np.zeros((r, H), np.uint16) for r in rows[sl]]
            prob.backward_bf16(hg, want)
            for a, b in zip(g_sg[sl], want):
                assert np.array_equal(_to_host_bits(a), b), (e, m)
            o_acc = [t.numpy().copy() for t in acc0[sl]]
            prob.backward_accumulate(hg, o_acc)
            for a, b in zip(g_acc[sl], o_acc):
                assert np.array_equal(a.cpu().numpy().view(np.uint32), b.view(np.uint32)), (e, m)
        base += per_map * n_maps
    for j in range(n_dst * n_maps):
        assert np.array_equal(_to_host_bits(g_dst[j]), o_dst[j]), j
    plan.close()


@pytest.mark.parametrize("hidden,tile", [(600, 1024), (600, 4096), (2048, 1024), (1536, 2048), (520, 1024), (4096, 8192)])
def test_sbh_rows_at_least_a_tile_long(hidden, tile):
    """[S, B, H] destination order with two samples per rank: rows are strided on
    the destination side.  Rows of at least a tile are cut into dense pieces
    (including a short last piece), shorter ones are grouped."""
    from parity import check_case_extended
    rng = np.random.default_rng(hidden + tile)
    tm = wl.token_map_from_lens(rng, 4, 96, hidden, [[5, 17, 9], [30], [], [12, 40]])
    src = wl.Grid(tp=2, dp=3)
    dst = wl.Grid(tp=2, cp=2, dp=2, cp_split=wl.CP_ZIGZAG, row_order=wl.ROW_SBH)
    hp.hp_set_option("tile_bytes_fwd", tile)
    hp.hp_set_option("tile_bytes_bwd", tile)
    check_case(src, dst, tm, seed=hidden)
    check_case_extended(src, dst, tm, seed=hidden)
    check_case_extended(src, dst, replace(tm, dtype=wl.DT_F32), seed=hidden + 1)


@pytest.mark.parametrize("row_order", [wl.ROW_BSH, wl.ROW_SBH])
def test_very_long_rows(row_order):
    """2 MiB rows (hidden 2^20): every tile lies inside one row; with [S,B,H]
    order and two samples per rank the rows are cut into dense pieces."""
    H = 1 << 20
    tm = wl.TokenMap(2, 8, H, [0, 1, 1], [1, 0, 5], [3, 2, 3])
    check_case(wl.Grid(tp=2, dp=2), wl.Grid(tp=2, cp=2, cp_split=wl.CP_ZIGZAG, row_order=row_order), tm, seed=9,
               gen_device="cuda")


def test_one_plan_from_several_threads_and_streams():
    """A plan is immutable after creation: four host threads, each with its own
    stream and buffers, run forward and backward on the same plan at once."""
    import threading
    w = wl.scaled(wl.long_context(n_images=12), 512)
    tm = w.maps[0]
    plan = hp.hp_plan_create(w.src, w.dst, tm)
    prob = oracle.Problem(w.src, w.dst, tm)
    sets, errors = [], []
    for k in range(4):
        src, pre, grads = make_inputs(prob, 50 + k, "cuda")
        sets.append(dict(src=src, pre=pre, dst=[t.clone() for t in pre], grads=grads,
                         sg=[torch.zeros_like(t) for t in src], stream=torch.cuda.Stream()))
    torch.cuda.synchronize()

    def work(s):
        try:
            for _ in range(5):
                hp.hp_forward(plan, s["src"], s["dst"], s["stream"])
                hp.hp_backward(plan, s["grads"], s["sg"], s["stream"])
            s["stream"].synchronize()
        except Exception as e:                      # noqa: BLE001 - reported below
            errors.append(repr(e))

    threads = [threading.Thread(target=work, args=(s,)) for s in sets]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for s in sets:
        want = [_to_host_bits(t).copy() for t in s["pre"]]
        prob.forward([_to_host_bits(t) for t in s["src"]], want)
        assert all(np.array_equal(_to_host_bits(a), b) for a, b in zip(s["dst"], want))
        o_sg = [np.zeros((r, 512), np.uint16) for r in prob.src_rows()]
        prob.backward_bf16([_to_host_bits(t) for t in s["grads"]], o_sg)
        assert all(np.array_equal(_to_host_bits(a), b) for a, b in zip(s["sg"], o_sg))
    plan.close()                                    # records one event on each of the four streams
    hp.hp_plan_create(w.src, w.dst, tm).close()


def test_readme_example_runs_as_written():
    """The calls of the README's usage section, with its grids and token map."""
    from paper_2605_27678_amd import Grid, TokenMap
    src = Grid(tp=1, dp=8)
    dst = Grid(tp=4, cp=8, dp=1, cp_split=1)
    tm = TokenMap(batch=1, seq=131072, hidden=5120,
                  img_sample=[0, 0], img_start=[100, 9000], img_len=[576, 2304])
    plan = hp.hp_plan_create(src, dst, tm)
    rows, drows = plan.src_rows(), plan.info.dst_rows_per_buf
    assert sum(rows) == 2880 and drows == 16384 and plan.info.n_dst_bufs == 32
    src_bufs = [wl.random_bf16((r, 5120), 3 + i, "cuda") for i, r in enumerate(rows)]
    dst_bufs = [torch.zeros((drows, 5120), dtype=torch.bfloat16, device="cuda") for _ in range(32)]
    dst_grads = [torch.ones((drows, 5120), dtype=torch.bfloat16, device="cuda") for _ in range(32)]
    src_grads = [torch.empty_like(t) for t in src_bufs]
    stream = torch.cuda.current_stream()
    hp.hp_plan_tune(plan, src_bufs, dst_bufs, dst_grads, src_grads)
    hp.hp_forward(plan, src_bufs, dst_bufs, stream)
    hp.hp_backward(plan, dst_grads, src_grads, stream)
    torch.cuda.synchronize()
    assert all(bool((g == 4).all()) for g in src_grads if g.numel())          # all-ones gradients return TP_dst
    written = sum(int((d != 0).any(dim=1).sum()) for d in dst_bufs)
    assert written == 4 * 2880                                                # image rows only, in all four replicas
