"""hp_forward_static (the entry point for callers that cannot allocate) against
hp_forward, through the C ABI: same inputs, same bits, on two calls in a row -
the second with a smaller input, so that tables left over from the first call
would show - plus the oracle, a host-only plan, a HIP-graph capture of the call
and the size limit."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import paper_2605_27678_amd as hp
from oracle import oracle
from paper_2605_27678_amd import binding
from paper_2605_27678_amd import workloads as wl
from parity import _to_host_bits

pytestmark = pytest.mark.gpu


def _run_both(w, tm, seed, host_only=True):
    """Forward through hp_forward (device plan) and hp_forward_static (host-only
    plan) into separate copies of the same prefilled destination buffers."""
    dev = "cuda:0"
    H = tm.hidden
    ref_plan = hp.hp_plan_create(w.src, w.dst, tm)
    st_plan = hp.hp_plan_create_host(w.src, w.dst, tm) if host_only else ref_plan
    assert st_plan.info.on_device == (0 if host_only else 1)
    rows, drows = ref_plan.src_rows(), ref_plan.info.dst_rows_per_buf
    src = [wl.random_bf16((r, H), seed * 100 + i, dev) for i, r in enumerate(rows)]
    pre = [wl.random_bf16((drows, H), seed * 100 + 40 + j, dev) for j in range(ref_plan.info.n_dst_bufs)]
    a = [t.clone() for t in pre]
    b = [t.clone() for t in pre]
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    hp.hp_forward(ref_plan, src, a, st)
    hp.hp_forward_static(st_plan, src, b, st)
    st.synchronize()
    for j, (x, y) in enumerate(zip(a, b)):
        assert torch.equal(x.view(torch.int16), y.view(torch.int16)), f"destination buffer {j} differs from hp_forward's"
    # and against the oracle (whole buffers: text rows untouched)
    prob = oracle.Problem(w.src, w.dst, tm)
    o = [_to_host_bits(t).copy() for t in pre]
    prob.forward([_to_host_bits(t) for t in src], o)
    for j in range(prob.n_dst):
        assert np.array_equal(_to_host_bits(b[j]), o[j]), f"destination buffer {j} differs from the oracle"
    if host_only:
        st_plan.close()
    ref_plan.close()


def test_static_forward_equals_forward_on_two_calls_the_second_smaller():
    big = wl.scaled(wl.long_context(), 640)                     # 34 segments, 32 destination buffers
    _run_both(big, big.maps[0], seed=1)
    small = wl.tiny()                                           # fewer segments, other grids: stale tables would show
    _run_both(small, small.maps[0], seed=2)
    one = wl.scaled(wl.long_context(n_images=1), 64)            # a single image
    _run_both(one, one.maps[0], seed=3)
    _run_both(big, big.maps[0], seed=4, host_only=False)        # a device plan is accepted as well


def test_static_forward_other_modes_and_launch_shapes():
    rng = np.random.default_rng(5)
    for i in range(6):
        src, dst, tm = wl.random_layout_case(rng)
        if i % 2 and (tm.seq // dst.cp) % dst.tp == 0:
            dst = replace(dst, tp_mode=wl.TP_SEQ_SHARD)
        w = wl.Workload("random", src, dst, [tm], 0)
        _run_both(w, tm, seed=10 + i)
    # several tree levels and another tile size: 300 one-row images -> 300 segments
    n = 300
    tm = wl.TokenMap(1, 4 * n, 128, [0] * n, [4 * i for i in range(n)], [1] * n)
    w = wl.Workload("many", wl.Grid(dp=3), wl.Grid(tp=2, cp=2, cp_split=wl.CP_ZIGZAG), [tm], 0)
    for tile in (1024, 4096):
        hp.hp_set_option("tile_bytes_fwd", tile)
        try:
            _run_both(w, tm, seed=30)
        finally:
            hp.hp_set_option("tile_bytes_fwd", -1)


def test_static_forward_rejects_tables_beyond_its_array():
    n = 4096                                                    # 4096 segments x 32 B > 64 KiB
    tm = wl.TokenMap(1, 2 * n, 8, [0] * n, [2 * i for i in range(n)], [1] * n)
    plan = hp.hp_plan_create_host(wl.Grid(), wl.Grid(), tm)
    assert plan.info.n_segments == n
    src = [torch.zeros((n, 8), dtype=torch.bfloat16, device="cuda")]
    dst = [torch.zeros((2 * n, 8), dtype=torch.bfloat16, device="cuda")]
    with pytest.raises(hp.HpError) as e:
        hp.hp_forward_static(plan, src, dst)
    assert e.value.code == binding.HP_ELAYOUT
    plan.close()
    # an empty plan is a no-op, as for hp_forward
    empty = hp.hp_plan_create_host(wl.Grid(), wl.Grid(), wl.TokenMap(1, 8, 8, [], [], []))
    hp.hp_forward_static(empty, [None], [torch.zeros((8, 8), dtype=torch.bfloat16, device="cuda")])
    empty.close()


def test_static_forward_can_be_captured_and_replayed():
    w = wl.scaled(wl.long_context(), 128)
    tm = w.maps[0]
    plan = hp.hp_plan_create_host(w.src, w.dst, tm)
    ref = hp.hp_plan_create(w.src, w.dst, tm)
    rows, drows = plan.src_rows(), plan.info.dst_rows_per_buf
    src = [wl.random_bf16((r, 128), 70 + i, "cuda") for i, r in enumerate(rows)]
    pre = [wl.random_bf16((drows, 128), 80 + j, "cuda") for j in range(32)]
    want = [t.clone() for t in pre]
    got = [t.clone() for t in pre]
    torch.cuda.synchronize()
    hp.hp_forward(ref, src, want)
    torch.cuda.synchronize()
    hp.hp_forward_static(plan, src, got)                        # first call on the device: outside the capture
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(g, stream=st):
        hp.hp_forward_static(plan, src, got, torch.cuda.current_stream())
    plan.close()                                                # the graph keeps the tables in its kernel arguments
    for rep in range(3):
        for t, p0 in zip(got, pre):
            t.copy_(p0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for j in range(32):
            assert torch.equal(got[j].view(torch.int16), want[j].view(torch.int16)), (rep, j)
    ref.close()
