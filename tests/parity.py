"""Shared driver of the GPU parity tests: same seeded inputs through the HIP
library (via its C ABI) and through the CPU oracle, compared element by
element as raw 16-bit patterns."""
from __future__ import annotations

import numpy as np
import torch

import paper_2605_27678_amd as hp
from oracle import oracle
from paper_2605_27678_amd import workloads as wl

SENTINEL_GPU = 0x7FC5      # bf16 NaN patterns no computation here produces
SENTINEL_CPU = 0x7FC9


def _bits_cpu(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def _to_host_bits(t: torch.Tensor) -> np.ndarray:
    return _bits_cpu(t.cpu())


def make_inputs(prob: oracle.Problem, seed: int, gen_device: str):
    """Source activations (TP copies other than 0 hold different data on
    purpose: forward must read the leader copy only), destination prefill
    ("text embeddings") and destination gradients (every replica different)."""
    H = prob.hidden
    rows = prob.src_rows()
    tp = prob.src_grid.tp
    src = []
    for i, r in enumerate(rows):
        s = seed * 1000 + i                                  # distinct per copy
        src.append(wl.random_bf16((r, H), s, gen_device))
    dst_rows = prob.dst_rows()
    pre = [wl.random_bf16((dst_rows, H), seed * 1000 + 300 + j, gen_device) for j in range(prob.n_dst)]
    grads = [wl.random_bf16((dst_rows, H), seed * 1000 + 600 + j, gen_device) for j in range(prob.n_dst)]
    return src, pre, grads


def check_case(src_grid, dst_grid, tm, seed=1, gen_device="cpu", stream=None, check_backward=True,
               grads_override=None, expect_launch=None):
    """Runs forward and backward on both sides and asserts bit equality.
    Returns the plan info.  expect_launch: the (forward, backward) launch
    shapes the new plan must start from."""
    dev = "cuda:0"
    plan = hp.hp_plan_create(src_grid, dst_grid, tm)
    if expect_launch is not None:
        assert (plan.get_launch(0), plan.get_launch(1)) == expect_launch
    prob = oracle.Problem(src_grid, dst_grid, tm)
    assert plan.src_rows() == prob.src_rows()
    assert plan.info.dst_rows_per_buf == prob.dst_rows()
    src, pre, grads = make_inputs(prob, seed, gen_device)
    if grads_override is not None:
        grads = grads_override
    st = stream if stream is not None else torch.cuda.current_stream()

    # ---- forward ----
    g_src = [t.to(dev) for t in src]
    g_dst = [t.to(dev).clone() for t in pre]
    torch.cuda.synchronize()
    hp.hp_forward(plan, g_src, g_dst, st)
    torch.cuda.synchronize()
    h_src = [_to_host_bits(t) for t in src]
    o_dst = [_to_host_bits(t).copy() for t in pre]
    prob.forward(h_src, o_dst)
    for j in range(prob.n_dst):
        got = _to_host_bits(g_dst[j])
        assert np.array_equal(got, o_dst[j]), f"forward mismatch in destination buffer {j}"
    del g_dst, o_dst, pre

    # ---- backward ----
    if check_backward:
        g_grads = [t.to(dev) for t in grads]
        g_sg = [torch.full((r, prob.hidden), 0, dtype=torch.int16, device=dev).fill_(SENTINEL_GPU).view(torch.bfloat16)
                for r in prob.src_rows()]
        torch.cuda.synchronize()
        hp.hp_backward(plan, g_grads, g_sg, st)
        torch.cuda.synchronize()
        h_grads = [_to_host_bits(t) for t in grads]
        o_sg = [np.full((r, prob.hidden), SENTINEL_CPU, np.uint16) for r in prob.src_rows()]
        prob.backward_bf16(h_grads, o_sg)
        for i in range(prob.n_src):
            got = _to_host_bits(g_sg[i])
            if not np.array_equal(got, o_sg[i]):
                # NaN results may differ in payload only
                a_nan = ((got & 0x7F80) == 0x7F80) & ((got & 0x7F) != 0)
                b_nan = ((o_sg[i] & 0x7F80) == 0x7F80) & ((o_sg[i] & 0x7F) != 0)
                same = (got == o_sg[i]) | (a_nan & b_nan)
                assert same.all(), f"backward mismatch in source buffer {i}"
                assert not np.any(got == SENTINEL_GPU), f"source buffer {i} has unwritten rows"
    info = plan.info
    plan.close()
    return info


def check_case_extended(src_grid, dst_grid, tm, seed=1, acc_launch=None):
    """binary32 payloads (forward, backward) and the accumulating backward for
    the token map's dtype, bit for bit against the oracle.  acc_launch: launch
    shape for hp_backward_accumulate instead of the default."""
    dev = "cuda:0"
    is_f32 = tm.dtype == wl.DT_F32
    tdt, ndt = (torch.float32, np.float32) if is_f32 else (torch.bfloat16, np.uint16)
    plan = hp.hp_plan_create(src_grid, dst_grid, tm)
    if acc_launch is not None:
        plan.set_launch(2, **acc_launch)
    prob = oracle.Problem(src_grid, dst_grid, tm)
    H, rows, drows = tm.hidden, prob.src_rows(), prob.dst_rows()

    def rnd(shape, s):
        g = torch.Generator().manual_seed(s)
        e = torch.randint(-10, 10, shape, generator=g).float()
        return (torch.randn(shape, generator=g) * torch.exp2(e)).to(tdt)

    def host(t):
        t = t.cpu().contiguous()
        return t.numpy().copy() if is_f32 else t.view(torch.int16).numpy().view(np.uint16).copy()

    src = [rnd((r, H), seed * 31 + i) for i, r in enumerate(rows)]
    pre = [rnd((drows, H), seed * 31 + 100 + j) for j in range(prob.n_dst)]
    grads = [rnd((drows, H), seed * 31 + 200 + j) for j in range(prob.n_dst)]
    acc0 = [torch.randn((r, H), generator=torch.Generator().manual_seed(seed * 31 + 300 + i)) for i, r in enumerate(rows)]

    g_dst = [t.to(dev) for t in pre]
    g_grads = [t.to(dev) for t in grads]
    if is_f32:                                              # the bf16 forward/backward are covered by check_case
        hp.hp_forward(plan, [t.to(dev) for t in src], g_dst)
        g_sg = [torch.full((r, H), float("nan"), dtype=tdt, device=dev) for r in rows]
        hp.hp_backward(plan, g_grads, g_sg)
    g_acc = [t.to(dev) for t in acc0]
    hp.hp_backward_accumulate(plan, g_grads, g_acc)
    hp.hp_backward_accumulate(plan, g_grads, g_acc)          # twice: really read-modify-write
    torch.cuda.synchronize()

    if is_f32:
        o_dst = [host(t) for t in pre]
        prob.forward([host(t) for t in src], o_dst)
        for j in range(prob.n_dst):
            assert np.array_equal(host(g_dst[j]).view(np.uint32), o_dst[j].view(np.uint32)), f"f32 forward, buffer {j}"
        o_sg = [np.full((r, H), np.nan, np.float32) for r in rows]
        prob.backward_f32([host(t) for t in grads], o_sg)
        for i in range(prob.n_src):
            assert np.array_equal(host(g_sg[i]).view(np.uint32), o_sg[i].view(np.uint32)), f"f32 backward, buffer {i}"
    o_acc = [t.numpy().copy() for t in acc0]
    hg = [host(t) for t in grads]
    prob.backward_accumulate(hg, o_acc)
    prob.backward_accumulate(hg, o_acc)
    for i in range(prob.n_src):
        got = g_acc[i].cpu().numpy()
        assert np.array_equal(got.view(np.uint32), o_acc[i].view(np.uint32)), f"accumulate, buffer {i}"
    plan.close()
