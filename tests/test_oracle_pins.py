"""Pins for the CPU oracle: everything here runs without a GPU and checks the
oracle against things other than itself - hand-worked fixtures, a brute-force
"build the global tensors and slice them" formulation, library routines
(memcpy-like identity, torch.index_copy_, torch's bf16 cast, numpy float32
addition), closed forms and invariants."""
import json
import os
import struct

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2605_27678_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------
# brute force: materialise the global boundary tensor X and the global fused
# tensor, then cut the destination buffers out of it with array slicing.
# ----------------------------------------------------------------------------

def default_src_dp(k_images, dp):
    """Closed form of the balanced contiguous interval rule: image k is on
    rank ceil((k+1)*DP/K) - 1."""
    k = np.arange(k_images, dtype=np.int64)
    return (((k + 1) * dp + k_images - 1) // k_images - 1).astype(np.int32) if k_images else k.astype(np.int32)


def brute_sources(src, tm, X):
    """Split X (rows in global image order) into the source buffers."""
    dps = tm.img_src_dp if tm.img_src_dp is not None else default_src_dp(tm.n_images, src.dp)
    bounds = np.concatenate([[0], np.cumsum(tm.img_len.astype(np.int64))])
    bufs = []
    for d in range(src.dp):
        parts = [X[bounds[k]:bounds[k + 1]] for k in range(tm.n_images) if dps[k] == d]
        rows = np.concatenate(parts, axis=0) if parts else X[:0]
        for _ in range(src.tp):
            bufs.append(rows.copy())
    return bufs


def brute_slice(dst, tm, G):
    """Cut a global [B, S, ...] array into the destination buffers."""
    B, S = tm.batch, tm.seq
    bl = B // dst.dp
    out = []
    for dp in range(dst.dp):
        slab = G[dp * bl:(dp + 1) * bl]
        for cp in range(dst.cp):
            if dst.cp_split == wl.CP_CONTIGUOUS:
                sl = S // dst.cp
                loc = slab[:, cp * sl:(cp + 1) * sl]
            else:
                c = S // (2 * dst.cp)
                chunks = slab.reshape((bl, 2 * dst.cp, c) + G.shape[2:])
                loc = np.concatenate([chunks[:, cp], chunks[:, 2 * dst.cp - 1 - cp]], axis=1)
            for tp in range(dst.tp):
                piece = loc
                if dst.tp_mode == wl.TP_SEQ_SHARD:
                    w = loc.shape[1] // dst.tp
                    piece = loc[:, tp * w:(tp + 1) * w]
                if dst.row_order == wl.ROW_SBH:
                    piece = np.swapaxes(piece, 0, 1)
                out.append(np.ascontiguousarray(piece).reshape((-1,) + G.shape[2:]))
    # the loops above ran dp, cp, tp with tp innermost: index = tp + TP*(cp + CP*dp)
    return out


def brute_forward(src, dst, tm, X, text_value):
    H = X.shape[1]
    fused = np.full((tm.batch, tm.seq, H), text_value, dtype=X.dtype)
    is_img = np.zeros((tm.batch, tm.seq), dtype=bool)
    n = 0
    for k in range(tm.n_images):
        b, s, ln = int(tm.img_sample[k]), int(tm.img_start[k]), int(tm.img_len[k])
        fused[b, s:s + ln] = X[n:n + ln]
        is_img[b, s:s + ln] = True
        n += ln
    return brute_slice(dst, tm, fused), brute_slice(dst, tm, is_img)


def row_id_payload(n_rows, hidden):
    """X[n, h] = 64*n + h in uint16: every element names its own row/column."""
    assert hidden <= 64 and n_rows * 64 < 65536
    return (64 * np.arange(n_rows, dtype=np.uint32)[:, None] + np.arange(hidden)[None, :]).astype(np.uint16)


def run_oracle_forward(src, dst, tm, X, text_value=0xFFFF):
    prob = oracle.Problem(src, dst, tm)
    srcs = brute_sources(src, tm, X)
    assert [a.shape[0] for a in srcs] == prob.src_rows()
    dsts = [np.full((prob.dst_rows(), tm.hidden), text_value, dtype=X.dtype) for _ in range(prob.n_dst)]
    prob.forward(srcs, dsts)
    return prob, srcs, dsts


# ----------------------------------------------------------------------------
# hand-worked fixture
# ----------------------------------------------------------------------------

def _grid_from(d, **kw):
    return wl.Grid(tp=d.get("tp", 1), cp=d.get("cp", 1), dp=d.get("dp", 1),
                   cp_split=wl.CP_ZIGZAG if d.get("cp_split") == "zigzag" else wl.CP_CONTIGUOUS,
                   row_order=wl.ROW_SBH if d.get("row_order") == "sbh" else wl.ROW_BSH, **kw)


def _bf16_bits(vals):
    return wl.bf16_bits(torch.tensor(vals, dtype=torch.float32).to(torch.bfloat16)).copy()


def test_worked_example_forward_and_backward():
    g = json.load(open(os.path.join(GOLDEN, "worked_example_zigzag.json")))
    src, dst = _grid_from(g["src"]), _grid_from(g["dst"])
    tm = wl.TokenMap(g["batch"], g["seq"], g["hidden"], g["img_sample"], g["img_start"], g["img_len"])
    prob = oracle.Problem(src, dst, tm)
    assert prob.src_rows() == [len(b) for b in g["src_bufs"]]
    srcs = [_bf16_bits(b).reshape(-1, 1) for b in g["src_bufs"]]
    dsts = [_bf16_bits([g["dst_text"]] * prob.dst_rows()).reshape(-1, 1) for _ in range(prob.n_dst)]
    prob.forward(srcs, dsts)
    for j in range(prob.n_dst):
        assert dsts[j].ravel().tolist() == _bf16_bits(g["dst_expected"][str(j)]).tolist(), j
    grads = [_bf16_bits(g["dst_grads"][str(j)]).reshape(-1, 1) for j in range(prob.n_dst)]
    sg = [np.full((r, 1), 0x7FC1, np.uint16) for r in prob.src_rows()]
    prob.backward_bf16(grads, sg)
    for i, exp in enumerate(g["src_grads_expected"]):
        assert sg[i].ravel().tolist() == _bf16_bits(exp).tolist(), i


def test_zigzag_positions_closed_form():
    """Rank r of C holds chunk r then chunk 2C-1-r; together the ranks tile
    [0, S) exactly once."""
    for C in (1, 2, 4, 8):
        S = 2 * C * 3
        tm = wl.TokenMap(1, S, 1, [0], [0], [S])          # one image covering everything
        src, dst = wl.Grid(), wl.Grid(cp=C, cp_split=wl.CP_ZIGZAG)
        prob = oracle.Problem(src, dst, tm)
        seen = []
        for r in range(C):
            _, rows = prob.forward_map(r)                 # source row == global position
            c = S // (2 * C)
            expect = list(range(r * c, (r + 1) * c)) + list(range((2 * C - 1 - r) * c, (2 * C - r) * c))
            assert rows.tolist() == expect
            seen += rows.tolist()
        assert sorted(seen) == list(range(S))


# ----------------------------------------------------------------------------
# brute force on many tiny layouts
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("seed", range(60))
def test_forward_matches_global_slicing(seed):
    rng = np.random.default_rng(1000 + seed)
    src, dst, tm = wl.random_layout_case(rng)
    X = row_id_payload(tm.n_rows, tm.hidden)
    prob, srcs, dsts = run_oracle_forward(src, dst, tm, X)
    want, is_img = brute_forward(src, dst, tm, X, 0xFFFF)
    assert len(want) == prob.n_dst
    for j in range(prob.n_dst):
        assert np.array_equal(dsts[j], want[j]), (seed, j)
    # bytes conserved: image rows over all destination buffers = TP_dst * N
    assert sum(int(m.sum()) for m in is_img) == dst.tp * tm.n_rows
    assert sum(a.shape[0] for a in srcs) == src.tp * tm.n_rows


@pytest.mark.parametrize("seed", range(20))
def test_forward_matches_global_slicing_spans_out_of_position_order(seed):
    """Images of a sample need not sit in the sequence in image order: the
    source keeps image order, the fused sequence follows the token map."""
    rng = np.random.default_rng(7000 + seed)
    src, dst, tm = wl.random_layout_case(rng)
    tm = wl.shuffle_spans(rng, tm)
    X = row_id_payload(tm.n_rows, tm.hidden)
    prob, srcs, dsts = run_oracle_forward(src, dst, tm, X)
    want, _ = brute_forward(src, dst, tm, X, 0xFFFF)
    for j in range(prob.n_dst):
        assert np.array_equal(dsts[j], want[j]), (seed, j)


def test_dense_reading_of_config_2_tiles_the_sequence():
    """8 images x 1024 tokens filling a sequence of 8192 with no text: every
    destination row is an image row, and sample b's slot p holds the image that
    the token map puts there."""
    w = wl.scaled(wl.colocated4_dense(), 4)
    tm = w.maps[0]
    assert tm.n_rows == tm.batch * tm.seq
    assert any(np.any(np.diff(tm.img_start[tm.img_sample == b]) < 0) for b in range(4))   # really out of order
    X = (np.arange(tm.n_rows, dtype=np.uint32)[:, None] * 4 + np.arange(4)[None, :]).astype(np.uint32)
    prob = oracle.Problem(w.src, w.dst, tm)
    srcs = brute_sources(w.src, tm, X)
    dsts = [np.full((prob.dst_rows(), 4), 0xFFFFFFFF, np.uint32) for _ in range(prob.n_dst)]
    prob.forward(srcs, dsts)
    want, is_img = brute_forward(w.src, w.dst, tm, X, 0xFFFFFFFF)
    for j in range(prob.n_dst):
        assert np.array_equal(dsts[j], want[j])
        assert is_img[j].all()
    # closed form: image k = 8 b + i sits at slot start/1024 of sample b
    d0 = dsts[0].reshape(4, 8, 1024, 4)
    for k in range(32):
        b, slot = int(tm.img_sample[k]), int(tm.img_start[k]) // 1024
        assert np.array_equal(d0[b, slot], X[1024 * k:1024 * (k + 1)])


@pytest.mark.parametrize("seed", range(20))
def test_forward_matches_global_slicing_seq_sharded(seed):
    rng = np.random.default_rng(5000 + seed)
    src, dst, tm = wl.random_layout_case(rng)
    from dataclasses import replace
    if (tm.seq // dst.cp) % dst.tp:
        dst = replace(dst, tp=2 if (tm.seq // dst.cp) % 2 == 0 else 1)
    dst = replace(dst, tp_mode=wl.TP_SEQ_SHARD)
    X = row_id_payload(tm.n_rows, tm.hidden)
    prob, srcs, dsts = run_oracle_forward(src, dst, tm, X)
    want, is_img = brute_forward(src, dst, tm, X, 0xFFFF)
    for j in range(prob.n_dst):
        assert np.array_equal(dsts[j], want[j]), (seed, j)
    assert sum(int(m.sum()) for m in is_img) == tm.n_rows       # nothing replicated


def test_paper_layout_pairs():
    """Layout pairs that appear in the paper (user configuration example: LLM
    TP4 DP2 with vision TP1 DP8 colocated, LLM TP2 with vision DP4 disjoint;
    bridge profile: encoder DP32 -> LLM DP16)."""
    pairs = [(wl.Grid(tp=1, dp=8), wl.Grid(tp=4, dp=2), 8, 4),
             (wl.Grid(tp=1, dp=4, rank_offset=4), wl.Grid(tp=2, dp=1), 4, 2),
             (wl.Grid(tp=1, dp=32), wl.Grid(tp=1, dp=16), 32, 1)]
    for src, dst, batch, imgs in pairs:
        rng = np.random.default_rng(7)
        tm = wl.token_map_from_lens(rng, batch, 24, 8, [[3] * imgs] * batch)
        X = row_id_payload(tm.n_rows, tm.hidden)
        prob, srcs, dsts = run_oracle_forward(src, dst, tm, X)
        want, _ = brute_forward(src, dst, tm, X, 0xFFFF)
        for j in range(prob.n_dst):
            assert np.array_equal(dsts[j], want[j])


def test_fan_in_two_quarter_shards_make_one_half_shard():
    """Figures 2 and 3: with B samples, source DP4 and destination DP2, source
    shards 0,1 (B/4 each) are concatenated in batch order into destination
    shard 0, shards 2,3 into shard 1; backward splits along the same
    intervals."""
    B, L = 4, 6
    tm = wl.TokenMap(B, L, 4, list(range(B)), [0] * B, [L] * B)   # all-image samples
    src, dst = wl.Grid(dp=4), wl.Grid(dp=2)
    X = row_id_payload(B * L, 4)
    prob, srcs, dsts = run_oracle_forward(src, dst, tm, X)
    assert prob.src_rows() == [L] * 4                      # equal B/4 batch intervals
    assert np.array_equal(dsts[0], np.concatenate([srcs[0], srcs[1]]))
    assert np.array_equal(dsts[1], np.concatenate([srcs[2], srcs[3]]))
    g = [row_id_payload(2 * L, 4) + np.uint16(j) for j in range(2)]   # any bf16 bit patterns, no NaN
    g = [np.where((x & 0x7F80) == 0x7F80, np.uint16(0), x) for x in g]
    sg = [np.zeros((L, 4), np.uint16) for _ in range(4)]
    prob.backward_bf16(g, sg)
    assert np.array_equal(sg[0], g[0][:L]) and np.array_equal(sg[1], g[0][L:])
    assert np.array_equal(sg[2], g[1][:L]) and np.array_equal(sg[3], g[1][L:])


def test_fan_out_dual_case():
    """Dual case of the figures: one B/2 source shard is split into two B/4
    destination shards; backward concatenates the sibling gradients."""
    B, L = 4, 5
    tm = wl.TokenMap(B, L, 4, list(range(B)), [0] * B, [L] * B)
    src, dst = wl.Grid(dp=2), wl.Grid(dp=4)
    X = row_id_payload(B * L, 4)
    prob, srcs, dsts = run_oracle_forward(src, dst, tm, X)
    assert prob.src_rows() == [2 * L] * 2
    for j in range(4):
        assert np.array_equal(dsts[j], srcs[j // 2][(j % 2) * L:(j % 2 + 1) * L])
    g = [np.full((L, 4), 0x3F80 + j, np.uint16) for j in range(4)]
    sg = [np.zeros((2 * L, 4), np.uint16) for _ in range(2)]
    prob.backward_bf16(g, sg)
    assert np.array_equal(sg[0], np.concatenate([g[0], g[1]]))
    assert np.array_equal(sg[1], np.concatenate([g[2], g[3]]))


def test_default_image_rule_reduces_to_equal_batch_intervals():
    """With a constant number of images per sample and DP dividing B, the
    image-unit rule is the paper's equal batch intervals: sample b is on source
    rank b // (B/DP)."""
    B, per, dp = 8, 3, 4
    rng = np.random.default_rng(3)
    tm = wl.token_map_from_lens(rng, B, 40, 8, [[4] * per] * B)
    prob = oracle.Problem(wl.Grid(dp=dp), wl.Grid(), tm)
    L = oracle.lib()
    import ctypes as C
    for k in range(tm.n_images):
        d = L.orc_image_src_dp(C.byref(prob.src), C.byref(prob.map), C.c_int32(k))
        assert d == int(tm.img_sample[k]) // (B // dp)
    # ragged counts: closed form of the same interval rule, ranks may be empty
    for K, dpn in [(5, 2), (3, 8), (31, 8), (1, 4), (7, 7)]:
        tm2 = wl.TokenMap(1, 4 * K, 8, [0] * K, [4 * i for i in range(K)], [4] * K)
        p2 = oracle.Problem(wl.Grid(dp=dpn), wl.Grid(), tm2)
        got = [L.orc_image_src_dp(C.byref(p2.src), C.byref(p2.map), C.c_int32(k)) for k in range(K)]
        assert got == default_src_dp(K, dpn).tolist()
        assert got == sorted(got) and all(0 <= d < dpn for d in got)


def test_identity_layout_is_memcpy():
    tm = wl.TokenMap(1, 37, 24, [0], [0], [37])
    X = np.random.default_rng(0).integers(0, 65536, size=(37, 24), dtype=np.uint16)
    prob, srcs, dsts = run_oracle_forward(wl.Grid(), wl.Grid(), tm, X)
    assert dsts[0].tobytes() == X.tobytes()


def test_single_sample_equals_index_copy():
    """No CP, one sample: forward is torch.index_copy_ of X into the sequence at
    the image positions."""
    rng = np.random.default_rng(11)
    tm = wl.token_map_from_lens(rng, 1, 200, 16, [[7, 30, 1, 19]])
    X = rng.integers(0, 30000, size=(tm.n_rows, 16)).astype(np.int16)
    prob, srcs, dsts = run_oracle_forward(wl.Grid(dp=3), wl.Grid(tp=2), tm, X.view(np.uint16), text_value=5)
    pos = np.concatenate([np.arange(s, s + l) for s, l in zip(tm.img_start, tm.img_len)])
    seq = torch.full((200, 16), 5, dtype=torch.int16)
    seq.index_copy_(0, torch.from_numpy(pos), torch.from_numpy(X))
    for j in range(2):
        assert np.array_equal(dsts[j].view(np.int16), seq.numpy())


def test_other_element_sizes_move_bit_for_bit():
    rng = np.random.default_rng(5)
    src, dst, tm = wl.random_layout_case(rng)
    for dt in (np.uint8, np.uint32, np.float64):
        X = rng.integers(0, 255, size=(tm.n_rows, tm.hidden)).astype(dt)
        prob = oracle.Problem(src, dst, tm)
        srcs = brute_sources(src, tm, X)
        dsts = [np.full((prob.dst_rows(), tm.hidden), 77, dtype=dt) for _ in range(prob.n_dst)]
        prob.forward(srcs, dsts)
        want, _ = brute_forward(src, dst, tm, X, 77)
        for j in range(prob.n_dst):
            assert np.array_equal(dsts[j], want[j])


# ----------------------------------------------------------------------------
# invariants
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("seed", range(25))
def test_forward_map_is_injective_and_invertible(seed):
    """Restricted to one TP replica, forward is a bijection between the image
    rows of the source side and the image rows of the destination side;
    applying the inverse after it gives the identity."""
    rng = np.random.default_rng(2000 + seed)
    src, dst, tm = wl.random_layout_case(rng)
    prob = oracle.Problem(src, dst, tm)
    pairs = {}
    for j in range(0, prob.n_dst, dst.tp):                # replica tp = 0 of every slice
        sb, sr = prob.forward_map(j)
        for t in range(1, dst.tp):                        # replicas agree
            sb2, sr2 = prob.forward_map(j + t)
            assert np.array_equal(sb, sb2) and np.array_equal(sr, sr2)
        for r in np.nonzero(sb >= 0)[0]:
            key = (int(sb[r]), int(sr[r]))
            assert key not in pairs                       # injective
            pairs[key] = (j, int(r))
    rows = prob.src_rows()
    want = {(i, r) for i in range(0, prob.n_src, src.tp) for r in range(rows[i])}
    assert set(pairs) == want                             # onto the source rows
    # inverse after forward = identity, shown on data
    X = row_id_payload(tm.n_rows, tm.hidden)
    srcs = brute_sources(src, tm, X)
    dsts = [np.zeros((prob.dst_rows(), tm.hidden), np.uint16) for _ in range(prob.n_dst)]
    prob.forward(srcs, dsts)
    back = [np.zeros_like(a) for a in srcs]
    for (i, r), (j, q) in pairs.items():
        back[i][r] = dsts[j][q]
    for i in range(0, prob.n_src, src.tp):
        assert np.array_equal(back[i], srcs[i])


def test_text_rows_untouched():
    rng = np.random.default_rng(42)
    src, dst, tm = wl.random_layout_case(rng)
    prob = oracle.Problem(src, dst, tm)
    X = row_id_payload(tm.n_rows, tm.hidden)
    srcs = brute_sources(src, tm, X)
    pre = [rng.integers(0, 65536, size=(prob.dst_rows(), tm.hidden), dtype=np.uint16) for _ in range(prob.n_dst)]
    dsts = [p.copy() for p in pre]
    prob.forward(srcs, dsts)
    for j in range(prob.n_dst):
        sb, _ = prob.forward_map(j)
        assert np.array_equal(dsts[j][sb < 0], pre[j][sb < 0])


# ----------------------------------------------------------------------------
# backward
# ----------------------------------------------------------------------------

def _f2b(x):
    return wl.bf16_bits(torch.as_tensor(x, dtype=torch.float32).to(torch.bfloat16)).copy()


def _b2f(bits):
    return wl.bits_to_bf16(bits).to(torch.float32).numpy()


@pytest.mark.parametrize("seed", range(15))
def test_all_ones_gradient_returns_replica_count(seed):
    rng = np.random.default_rng(3000 + seed)
    src, dst, tm = wl.random_layout_case(rng)
    prob = oracle.Problem(src, dst, tm)
    g = [_f2b(np.ones((prob.dst_rows(), tm.hidden), np.float32)) for _ in range(prob.n_dst)]
    sg = [np.full((r, tm.hidden), 0x7FC1, np.uint16) for r in prob.src_rows()]
    prob.backward_bf16(g, sg)
    for a in sg:
        assert np.array_equal(_b2f(a), np.full(a.shape, float(dst.tp), np.float32))


@pytest.mark.parametrize("seed", range(15))
def test_backward_is_adjoint_of_forward(seed):
    """<forward(x), g> over image rows == <x, backward(g)> with small-integer
    values, for which every sum is exact in bf16/binary32."""
    rng = np.random.default_rng(4000 + seed)
    src, dst, tm = wl.random_layout_case(rng)
    prob = oracle.Problem(src, dst, tm)
    Xf = rng.integers(-8, 9, size=(tm.n_rows, tm.hidden)).astype(np.float32)
    srcs = brute_sources(src, tm, _f2b(Xf))
    dsts = [_f2b(np.zeros((prob.dst_rows(), tm.hidden), np.float32)) for _ in range(prob.n_dst)]
    prob.forward(srcs, dsts)
    gf = [rng.integers(-8, 9, size=(prob.dst_rows(), tm.hidden)).astype(np.float32) for _ in range(prob.n_dst)]
    sg = [np.full((r, tm.hidden), 0x7FC1, np.uint16) for r in prob.src_rows()]
    prob.backward_bf16([_f2b(x) for x in gf], sg)
    lhs = 0.0
    for j in range(prob.n_dst):
        sb, _ = prob.forward_map(j)
        lhs += float((_b2f(dsts[j]).astype(np.float64) * gf[j])[sb >= 0].sum())
    rhs = sum(float((_b2f(srcs[i]).astype(np.float64) * _b2f(sg[i])).sum())
              for i in range(0, prob.n_src, src.tp))
    assert lhs == rhs
    for i in range(0, prob.n_src, src.tp):                 # source TP replicas identical
        for t in range(1, src.tp):
            assert np.array_equal(sg[i], sg[i + t])


def test_backward_tp1_is_inverse_permutation():
    rng = np.random.default_rng(9)
    from dataclasses import replace
    for _ in range(10):
        src, dst, tm = wl.random_layout_case(rng)
        dst = replace(dst, tp=1)
        X = row_id_payload(tm.n_rows, tm.hidden) & np.uint16(0x3FFF)   # finite bf16 patterns
        prob, srcs, dsts = run_oracle_forward(src, dst, tm, X, text_value=0)
        sg = [np.full(a.shape, 0x7FC1, np.uint16) for a in srcs]
        prob.backward_bf16(dsts, sg)
        for a, b in zip(sg, srcs):
            assert np.array_equal(a, b)


def test_backward_tp2_is_one_rounded_add():
    """Two replicas: the fold is a single binary32 add (numpy float32) followed
    by torch's bf16 rounding."""
    rng = np.random.default_rng(10)
    tm = wl.token_map_from_lens(rng, 1, 64, 32, [[5, 9, 17]])
    src, dst = wl.Grid(dp=2), wl.Grid(tp=2, cp=2, cp_split=wl.CP_ZIGZAG)
    prob = oracle.Problem(src, dst, tm)
    scale = np.exp2(rng.integers(-20, 20, size=(prob.n_dst, prob.dst_rows(), 32))).astype(np.float32)
    gf = rng.standard_normal((prob.n_dst, prob.dst_rows(), 32)).astype(np.float32) * scale
    gb = [_f2b(gf[j]) for j in range(prob.n_dst)]
    sg = [np.zeros((r, 32), np.uint16) for r in prob.src_rows()]
    prob.backward_bf16(gb, sg)
    # expected through the forward map and library arithmetic
    for j in range(0, prob.n_dst, 2):
        sb, sr = prob.forward_map(j)
        s = (_b2f(gb[j]) + _b2f(gb[j + 1])).astype(np.float32)
        want = _f2b(s)
        for r in np.nonzero(sb >= 0)[0]:
            assert np.array_equal(sg[sb[r]][sr[r]], want[r])


def test_fixed_order_fold_and_rounding_fixture():
    g = json.load(open(os.path.join(GOLDEN, "bf16_rounding.json")))
    for case in g["round"]:
        f = struct.unpack("<f", struct.pack("<I", int(case["f32_hex"], 16)))[0]
        assert oracle.f32_to_bf16(f) == int(case["bf16_hex"], 16), case["why"]
        assert oracle.f32_bits_to_bf16(int(case["f32_hex"], 16)) == int(case["bf16_hex"], 16), case["why"]
    for case in g["fold"]:
        terms = case["terms"]
        tp = len(terms)
        tm = wl.TokenMap(1, 1, 1, [0], [0], [1])
        prob = oracle.Problem(wl.Grid(), wl.Grid(tp=tp), tm)
        grads = [_f2b([[t]]) for t in terms]
        assert [float(_b2f(x)[0, 0]) for x in grads] == [float(t) for t in terms]   # representable
        sg = [np.zeros((1, 1), np.uint16)]
        prob.backward_bf16(grads, sg)
        assert float(_b2f(sg[0])[0, 0]) == float(case["result"]), case["why"]


def test_bf16_rounding_matches_torch_cast():
    rng = np.random.default_rng(77)
    bits = rng.integers(0, 2 ** 32, size=20000, dtype=np.uint64).astype(np.uint32)
    f = bits.view(np.float32)
    t = torch.from_numpy(f.copy()).to(torch.bfloat16)
    want = wl.bf16_bits(t)
    for x, u, w in zip(f.tolist()[:4000], bits.tolist()[:4000], want.tolist()[:4000]):
        got = oracle.f32_bits_to_bf16(u)
        if x == x:
            assert got == oracle.f32_to_bf16(x)
        if x != x:
            assert (got & 0x7F80) == 0x7F80 and (got & 0x7F) != 0      # NaN stays NaN
        else:
            assert got == w
    for h in rng.integers(0, 65536, size=500).tolist():
        v = oracle.bf16_to_f32(h)
        w = wl.bits_to_bf16(np.array([h], np.uint16)).to(torch.float32).item()
        assert (v != v and w != w) or v == w


def test_backward_subnormals_are_kept():
    """Two bf16 subnormals add to a binary32 subnormal that must not be flushed."""
    tm = wl.TokenMap(1, 1, 1, [0], [0], [1])
    prob = oracle.Problem(wl.Grid(), wl.Grid(tp=2), tm)
    a = np.array([[0x0001]], np.uint16)      # smallest bf16 subnormal, 2^-133
    b = np.array([[0x0002]], np.uint16)
    sg = [np.zeros((1, 1), np.uint16)]
    prob.backward_bf16([a, b], sg)
    assert int(sg[0][0, 0]) == 0x0003


def test_backward_ignores_text_rows_and_writes_every_source_row():
    rng = np.random.default_rng(12)
    for _ in range(10):
        src, dst, tm = wl.random_layout_case(rng)
        prob = oracle.Problem(src, dst, tm)
        g = [_f2b(rng.integers(-4, 5, size=(prob.dst_rows(), tm.hidden)).astype(np.float32))
             for _ in range(prob.n_dst)]
        sg1 = [np.full((r, tm.hidden), 0x7FC1, np.uint16) for r in prob.src_rows()]
        prob.backward_bf16(g, sg1)
        assert all(not np.any(a == 0x7FC1) for a in sg1)             # every row overwritten
        g2 = [x.copy() for x in g]
        for j in range(prob.n_dst):
            sb, _ = prob.forward_map(j)
            g2[j][sb < 0] = 0x7FC0                                   # poison text-row grads
        sg2 = [np.zeros((r, tm.hidden), np.uint16) for r in prob.src_rows()]
        prob.backward_bf16(g2, sg2)
        for a, b in zip(sg1, sg2):
            assert np.array_equal(a, b)


def test_named_workloads_have_the_stated_shapes():
    w = wl.tiny()
    assert (w.maps[0].batch, w.maps[0].seq, w.maps[0].hidden, w.maps[0].n_rows) == (2, 320, 64, 128)
    w = wl.colocated4()
    assert (w.maps[0].seq, w.maps[0].n_rows) == (16384, 32768)
    w = wl.long_context()
    m = w.maps[0]
    assert m.seq == 131072 and m.hidden == 5120 and 0.30 * m.seq <= m.n_rows <= 0.30 * m.seq + 2304
    assert 1 <= m.n_images <= 32 and m.img_len.min() >= 256 and m.img_len.max() <= 2304
    w = wl.non_colocated()
    assert len(w.maps) == 16 and all(4 <= x.n_images <= 16 and set(x.img_len) == {576} for x in w.maps)
    w = wl.large_scale()
    m = w.maps[0]
    assert m.seq == 65536 and m.n_rows >= 32768 and m.img_len.min() >= 64 and m.img_len.max() <= 4096
    for w in (wl.tiny(), wl.colocated4(), wl.long_context(), wl.large_scale()):
        for m in w.maps:                                   # spans never overlap, stay in range
            for b in range(m.batch):
                sel = m.img_sample == b
                s, l = m.img_start[sel].astype(np.int64), m.img_len[sel].astype(np.int64)
                o = np.argsort(s)
                assert np.all(s[o][1:] >= (s[o] + l[o])[:-1]) and np.all(s + l <= m.seq) and np.all(s >= 0)


# ----------------------------------------------------------------------------
# binary32 gradients and accumulating output
# ----------------------------------------------------------------------------

def test_generic_backward_agrees_with_the_bf16_backward():
    """orc_backward(dtype=bf16, overwrite) is the same computation as
    orc_backward_bf16 (which the fixtures above pin)."""
    rng = np.random.default_rng(21)
    for _ in range(10):
        src, dst, tm = wl.random_layout_case(rng)
        prob = oracle.Problem(src, dst, tm)
        e = rng.integers(-12, 12, size=(prob.n_dst, prob.dst_rows(), tm.hidden))
        g = [_f2b((rng.standard_normal((prob.dst_rows(), tm.hidden)) * np.exp2(e[j])).astype(np.float32))
             for j in range(prob.n_dst)]
        a = [np.full((r, tm.hidden), 0x7FC1, np.uint16) for r in prob.src_rows()]
        b = [np.full((r, tm.hidden), 0x7FC1, np.uint16) for r in prob.src_rows()]
        prob.backward_bf16(g, a)
        prob._backward(0, False, g, b)
        assert all(np.array_equal(x, y) for x, y in zip(a, b))


def test_f32_backward_fold_order_and_tp2_is_numpy_add():
    g = json.load(open(os.path.join(GOLDEN, "bf16_rounding.json")))
    tm = wl.TokenMap(1, 1, 1, [0], [0], [1])
    for case in g["fold"][:3]:                       # the order-sensitive binary32 cases
        terms = case["terms"]
        prob = oracle.Problem(wl.Grid(), wl.Grid(tp=len(terms)), tm)
        out = [np.zeros((1, 1), np.float32)]
        prob.backward_f32([np.array([[t]], np.float32) for t in terms], out)
        assert float(out[0][0, 0]) == float(case["result"]), case["why"]
    # no rounding to bf16: 1 + 2^-8 stays
    prob = oracle.Problem(wl.Grid(), wl.Grid(tp=2), tm)
    out = [np.zeros((1, 1), np.float32)]
    prob.backward_f32([np.array([[1.0]], np.float32), np.array([[2.0 ** -8]], np.float32)], out)
    assert float(out[0][0, 0]) == 1.00390625
    # two replicas on a random layout: one numpy float32 add, routed by the forward map
    rng = np.random.default_rng(22)
    tm = wl.token_map_from_lens(rng, 1, 64, 16, [[5, 9, 17]])
    src, dst = wl.Grid(tp=2, dp=2), wl.Grid(tp=2, cp=2, cp_split=wl.CP_ZIGZAG)
    prob = oracle.Problem(src, dst, tm)
    gf = [(rng.standard_normal((prob.dst_rows(), 16)) * np.exp2(rng.integers(-20, 20, size=(prob.dst_rows(), 16)))).astype(np.float32)
          for _ in range(prob.n_dst)]
    sg = [np.full((r, 16), np.nan, np.float32) for r in prob.src_rows()]
    prob.backward_f32(gf, sg)
    for j in range(0, prob.n_dst, 2):
        sb, sr = prob.forward_map(j)
        want = gf[j] + gf[j + 1]
        for r in np.nonzero(sb >= 0)[0]:
            for ts in range(2):
                assert np.array_equal(sg[sb[r] + ts][sr[r]], want[r])
    assert not any(np.isnan(a).any() for a in sg)


def test_accumulate_adds_the_fold_to_what_is_there():
    """acc_out = acc_in + fold(replicas): shown on small integers (exact), on a
    case where the extra add rounds (2^24 accumulator + 1), and applied twice."""
    rng = np.random.default_rng(23)
    for dtype in (0, 1):
        src, dst, tm = wl.random_layout_case(rng)
        prob = oracle.Problem(src, dst, tm)
        gi = [rng.integers(-8, 9, size=(prob.dst_rows(), tm.hidden)).astype(np.float32) for _ in range(prob.n_dst)]
        g = [_f2b(x) for x in gi] if dtype == 0 else gi
        start = [rng.integers(-50, 50, size=(r, tm.hidden)).astype(np.float32) for r in prob.src_rows()]
        acc = [a.copy() for a in start]
        prob.backward_accumulate(g, acc)
        once = [np.zeros_like(a) for a in start]
        (prob.backward_f32 if dtype == 1 else (lambda gg, out: prob._backward(0, True, gg, out)))(g, once)
        for a, s, o in zip(acc, start, once):
            assert np.array_equal(a, s + o)                  # integers: exact
        prob.backward_accumulate(g, acc)
        for a, s, o in zip(acc, start, once):
            assert np.array_equal(a, s + 2 * o)
    tm = wl.TokenMap(1, 1, 1, [0], [0], [1])
    prob = oracle.Problem(wl.Grid(), wl.Grid(tp=2), tm)
    acc = [np.array([[16777216.0]], np.float32)]
    prob.backward_accumulate([_f2b([[0.5]]), _f2b([[0.5]])], acc)     # fold = 1 exactly; 2^24 + 1 ties to even
    assert float(acc[0][0, 0]) == 16777216.0
    acc = [np.array([[16777216.0]], np.float32)]
    prob.backward_accumulate([_f2b([[1.0]]), _f2b([[1.0]])], acc)     # fold = 2; 2^24 + 2 is exact
    assert float(acc[0][0, 0]) == 16777218.0


# ----------------------------------------------------------------------------
# backward by "un-slicing": every destination-gradient buffer is put back into a
# global [B, S, H] gradient (one per TP copy), the copies are folded with numpy
# float32 adds, the result is rounded with torch's bf16 cast, and the image rows
# are read out in global image order and cut into the source buffers.  Nothing
# of the oracle is used; both destination TP modes.
# ----------------------------------------------------------------------------

def brute_backward(src, dst, tm, grads_f32):
    """grads_f32: one float32 [rows, H] array per destination buffer.  Returns
    the folded binary32 gradient of every source buffer (before any rounding)."""
    B, S, H = tm.batch, tm.seq, tm.hidden
    ids = np.arange(B * S, dtype=np.int64).reshape(B, S)
    where = brute_slice(dst, tm, ids)                     # global position of every local row
    n_copies = 1 if dst.tp_mode == wl.TP_SEQ_SHARD else dst.tp
    G = np.zeros((n_copies, B * S, H), np.float32)
    seen = np.zeros((n_copies, B * S), np.int32)
    for j, pos in enumerate(where):
        t = j % dst.tp if n_copies > 1 else 0
        G[t, pos] = grads_f32[j]
        seen[t, pos] += 1
    assert np.all(seen == 1)                              # every copy tiles the fused tensor exactly once
    fold = G[0].copy()
    for t in range(1, n_copies):                          # ascending tp, one IEEE binary32 add each
        fold = (fold + G[t]).astype(np.float32)
    img_pos = np.concatenate([int(b) * S + np.arange(int(s), int(s) + int(ln)) for b, s, ln in
                              zip(tm.img_sample, tm.img_start, tm.img_len)]) if tm.n_images \
        else np.zeros(0, np.int64)
    return brute_sources(src, tm, fold[img_pos])


def seq_shard_case(rng, tp=None):
    """A random small layout whose destination is sequence-sharded over `tp`
    ranks (drawn again until the CP-local sequence divides)."""
    from dataclasses import replace
    for _ in range(1000):
        src, dst, tm = wl.random_layout_case(rng)
        t = dst.tp if tp is None else tp
        if (tm.seq // dst.cp) % t == 0 and tm.n_images:
            return src, replace(dst, tp=t, tp_mode=wl.TP_SEQ_SHARD), tm
    raise AssertionError("no case drawn")


def wide_range_grads(rng, prob, hidden):
    e = rng.integers(-12, 12, size=(prob.n_dst, prob.dst_rows(), hidden))
    return [(rng.standard_normal((prob.dst_rows(), hidden)) * np.exp2(e[j])).astype(np.float32)
            for j in range(prob.n_dst)]


@pytest.mark.parametrize("mode", ["replicate", "seq_shard"])
@pytest.mark.parametrize("seed", range(12))
def test_backward_matches_global_unslicing(seed, mode):
    rng = np.random.default_rng(8000 + seed)
    if mode == "seq_shard":
        src, dst, tm = seq_shard_case(rng, tp=(2, 3, 4)[seed % 3])
    else:
        src, dst, tm = wl.random_layout_case(rng)
    prob = oracle.Problem(src, dst, tm)
    gb = [_f2b(x) for x in wide_range_grads(rng, prob, tm.hidden)]           # bf16 bit patterns
    want_f32 = brute_backward(src, dst, tm, [_b2f(x) for x in gb])
    want_bits = [_f2b(x) for x in want_f32]                                  # torch's rounding
    for call in (prob.backward_bf16, lambda g, out: prob._backward(0, False, g, out)):
        sg = [np.full((r, tm.hidden), 0x7FC1, np.uint16) for r in prob.src_rows()]
        call(gb, sg)
        for a, w in zip(sg, want_bits):
            assert np.array_equal(a, w), (seed, mode)
    # binary32 gradients: no rounding at the end
    gf = wide_range_grads(rng, prob, tm.hidden)
    want = brute_backward(src, dst, tm, gf)
    out = [np.full((r, tm.hidden), np.nan, np.float32) for r in prob.src_rows()]
    prob.backward_f32(gf, out)
    for a, w in zip(out, want):
        assert np.array_equal(a.view(np.uint32), w.view(np.uint32)), (seed, mode)
    # accumulating output: start + fold, one more binary32 add
    start = [rng.standard_normal((r, tm.hidden)).astype(np.float32) for r in prob.src_rows()]
    for g, w_fold in ((gb, want_f32), (gf, want)):
        acc = [a.copy() for a in start]
        prob.backward_accumulate(g, acc)
        for a, s0, w in zip(acc, start, w_fold):
            assert np.array_equal(a.view(np.uint32), (s0 + w).astype(np.float32).view(np.uint32)), (seed, mode)


@pytest.mark.parametrize("tp", [2, 3, 4])
def test_seq_sharded_backward_is_the_inverse_permutation_of_forward(tp):
    """Sequence-sharded TP replicates nothing, so there is nothing to sum:
    backward applied to forward's output returns the source bit for bit, and
    all-ones gradients come back as 1 (not TP_dst)."""
    rng = np.random.default_rng(8100 + tp)
    for _ in range(6):
        src, dst, tm = seq_shard_case(rng, tp=tp)
        X = row_id_payload(tm.n_rows, tm.hidden) & np.uint16(0x3FFF)          # finite, all different
        prob, srcs, dsts = run_oracle_forward(src, dst, tm, X, text_value=0x7FC0)
        for call in (prob.backward_bf16, lambda g, out: prob._backward(0, False, g, out)):
            sg = [np.full(a.shape, 0x7FC1, np.uint16) for a in srcs]
            call(dsts, sg)
            for a, b in zip(sg, srcs):
                assert np.array_equal(a, b)
        ones = [_f2b(np.ones((prob.dst_rows(), tm.hidden), np.float32)) for _ in range(prob.n_dst)]
        sg = [np.full(a.shape, 0x7FC1, np.uint16) for a in srcs]
        prob.backward_bf16(ones, sg)
        for a in sg:
            assert np.array_equal(_b2f(a), np.ones(a.shape, np.float32))
        of = [np.ones((prob.dst_rows(), tm.hidden), np.float32) for _ in range(prob.n_dst)]
        out = [np.full(a.shape, np.nan, np.float32) for a in srcs]
        prob.backward_f32(of, out)
        assert all(np.array_equal(a, np.ones_like(a)) for a in out)
        acc = [np.full(a.shape, 5.0, np.float32) for a in srcs]
        prob.backward_accumulate(of, acc)
        assert all(np.array_equal(a, np.full_like(a, 6.0)) for a in acc)


@pytest.mark.parametrize("seed", range(9))
def test_seq_sharded_backward_adjoint_and_text_rows(seed):
    rng = np.random.default_rng(8200 + seed)
    src, dst, tm = seq_shard_case(rng, tp=(2, 3, 4)[seed % 3])
    prob = oracle.Problem(src, dst, tm)
    Xf = rng.integers(-8, 9, size=(tm.n_rows, tm.hidden)).astype(np.float32)
    srcs = brute_sources(src, tm, _f2b(Xf))
    dsts = [_f2b(np.zeros((prob.dst_rows(), tm.hidden), np.float32)) for _ in range(prob.n_dst)]
    prob.forward(srcs, dsts)
    gf = [rng.integers(-8, 9, size=(prob.dst_rows(), tm.hidden)).astype(np.float32) for _ in range(prob.n_dst)]
    sg = [np.full((r, tm.hidden), 0x7FC1, np.uint16) for r in prob.src_rows()]
    prob.backward_bf16([_f2b(x) for x in gf], sg)
    lhs = 0.0
    for j in range(prob.n_dst):
        sb, _ = prob.forward_map(j)
        lhs += float((_b2f(dsts[j]).astype(np.float64) * gf[j])[sb >= 0].sum())
    rhs = sum(float((_b2f(srcs[i]).astype(np.float64) * _b2f(sg[i])).sum()) for i in range(0, prob.n_src, src.tp))
    assert lhs == rhs
    for i in range(0, prob.n_src, src.tp):
        for t in range(1, src.tp):
            assert np.array_equal(sg[i], sg[i + t])
    assert all(not np.any(a == 0x7FC1) for a in sg)                          # every source row written
    # gradients on text rows are ignored
    g2 = [_f2b(x) for x in gf]
    for j in range(prob.n_dst):
        sb, _ = prob.forward_map(j)
        g2[j][sb < 0] = 0x7FC0
    sg2 = [np.zeros((r, tm.hidden), np.uint16) for r in prob.src_rows()]
    prob.backward_bf16(g2, sg2)
    for a, b in zip(sg, sg2):
        assert np.array_equal(a, b)


def test_signalling_nan_stays_nan_when_rounded_to_bf16():
    """A NaN whose payload lies only in the 16 discarded bits must not round to
    infinity; the sign is kept."""
    g = json.load(open(os.path.join(GOLDEN, "bf16_rounding.json")))
    assert len(g["nan"]) >= 4
    for case in g["nan"]:
        got = oracle.f32_bits_to_bf16(int(case["f32_hex"], 16))   # as bits: a Python float would quiet the NaN
        assert (got & 0x7F80) == 0x7F80 and (got & 0x007F) != 0, case
        assert (got >> 15) == int(case["sign"]), case
    # and through the backward fold: a NaN gradient gives a NaN result
    tm = wl.TokenMap(1, 1, 1, [0], [0], [1])
    prob = oracle.Problem(wl.Grid(), wl.Grid(tp=2), tm)
    sg = [np.zeros((1, 1), np.uint16)]
    prob.backward_bf16([np.array([[0x7FA0]], np.uint16), np.array([[0x3F80]], np.uint16)], sg)
    assert (int(sg[0][0, 0]) & 0x7F80) == 0x7F80 and (int(sg[0][0, 0]) & 0x7F) != 0


# ----------------------------------------------------------------------------
# zeroing the inserted rows (gradient with respect to the text embeddings)
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("seed", range(16))
def test_zero_image_rows_matches_the_sliced_image_mask(seed):
    """Expected result by slicing: the global image mask cut into the destination
    buffers says which rows become zero; all other rows keep their content."""
    rng = np.random.default_rng(8300 + seed)
    if seed % 4 == 3:
        src, dst, tm = seq_shard_case(rng)
    else:
        src, dst, tm = wl.random_layout_case(rng)
    if seed % 5 == 4:
        tm = wl.shuffle_spans(rng, tm)
    prob = oracle.Problem(src, dst, tm)
    for dt in (np.uint16, np.float32):
        pre = [rng.integers(1, 60000, size=(prob.dst_rows(), tm.hidden)).astype(dt) for _ in range(prob.n_dst)]
        got = [p.copy() for p in pre]
        prob.zero_image_rows(got)
        _, is_img = brute_forward(src, dst, tm, np.zeros((tm.n_rows, tm.hidden), dt), 0)
        n_zeroed = 0
        for j in range(prob.n_dst):
            want = pre[j].copy()
            want[is_img[j]] = 0
            assert np.array_equal(got[j], want), (seed, j)
            n_zeroed += int(is_img[j].sum())
        assert n_zeroed == (1 if dst.tp_mode == wl.TP_SEQ_SHARD else dst.tp) * tm.n_rows


def test_zero_image_rows_is_the_text_gradient_of_the_fused_sequence():
    """torch autograd on the definition: fused = text with the image rows
    replaced; d(sum(fused * g))/d(text) is g with the image rows blanked."""
    rng = np.random.default_rng(8400)
    tm = wl.token_map_from_lens(rng, 1, 48, 8, [[5, 9, 3]])
    prob = oracle.Problem(wl.Grid(dp=2), wl.Grid(), tm)
    pos = torch.from_numpy(np.concatenate([np.arange(s, s + l) for s, l in zip(tm.img_start, tm.img_len)]))
    text = torch.randn(48, 8, requires_grad=True)
    X = torch.randn(tm.n_rows, 8, requires_grad=True)
    g = torch.randn(48, 8)
    fused = text.index_copy(0, pos, X)
    (fused * g).sum().backward()
    got = [g.numpy().copy()]
    prob.zero_image_rows(got)
    assert np.array_equal(got[0], text.grad.numpy())
    assert np.array_equal(X.grad.numpy(), g.numpy()[pos.numpy()])          # and the other half goes to the source
