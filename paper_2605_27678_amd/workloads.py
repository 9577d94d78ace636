"""Seeded synthetic inputs for the boundary layout transform.

This module only *describes* problems and draws random numbers: module grids,
token maps (where the image-token spans sit in the fused sequence) and random
bf16 tensors of a shape the caller names.  It contains none of the transform's
arithmetic (no rank decoding, no sequence split, no image-to-rank rule), so the
HIP library and the CPU oracle can both be fed from it without sharing any of
the method between them.

The five named workloads stand in for the paper's multimodal training inputs
(image/text samples with 576 projected tokens per image at hidden 4096 for the
LLaVA validation, 8K-128K fused sequences with 50-87.5 % vision tokens in the
throughput tables; appendix "LLaVA validation details" and Tables A2-A4).  Only
those shapes are used; every value is synthetic.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Optional, Sequence

import numpy as np

TP_REPLICATE = 0
TP_SEQ_SHARD = 1
CP_CONTIGUOUS = 0
CP_ZIGZAG = 1
ROW_BSH = 0
ROW_SBH = 1
DT_BF16 = 0
DT_F32 = 1

BASE_SEED = 276780


@dataclass(frozen=True)
class Grid:
    """One module's logical grid and first physical rank id (Method, first
    paragraph: layout G_m and rank set R_m; appendix "Open-source user
    configuration example": TP/PP/DP sizes plus rank_offset)."""
    tp: int = 1
    cp: int = 1
    dp: int = 1
    pp: int = 1
    rank_offset: int = 0
    tp_mode: int = TP_REPLICATE
    cp_split: int = CP_CONTIGUOUS
    row_order: int = ROW_BSH

    @property
    def n_ranks(self) -> int:
        return self.tp * self.cp * self.dp


@dataclass
class TokenMap:
    """Fused-sequence shape and the image spans inside it, in global image
    order (sample-major)."""
    batch: int
    seq: int
    hidden: int
    img_sample: np.ndarray
    img_start: np.ndarray
    img_len: np.ndarray
    img_src_dp: Optional[np.ndarray] = None
    dtype: int = DT_BF16

    def __post_init__(self):
        self.img_sample = np.ascontiguousarray(self.img_sample, dtype=np.int32)
        self.img_start = np.ascontiguousarray(self.img_start, dtype=np.int32)
        self.img_len = np.ascontiguousarray(self.img_len, dtype=np.int32)
        if self.img_src_dp is not None:
            self.img_src_dp = np.ascontiguousarray(self.img_src_dp, dtype=np.int32)

    @property
    def n_images(self) -> int:
        return int(self.img_len.shape[0])

    @property
    def n_rows(self) -> int:
        return int(self.img_len.astype(np.int64).sum())


@dataclass
class Workload:
    name: str
    src: Grid
    dst: Grid
    maps: List[TokenMap]          # one entry per microbatch
    seed: int
    note: str = ""


def place_spans(rng: np.random.Generator, seq: int, lens: Sequence[int]) -> np.ndarray:
    """Start positions for consecutive, non-overlapping spans of the given
    lengths inside [0, seq): the seq - sum(lens) text tokens are split into
    len(lens)+1 gaps by a uniform random composition (gaps may be empty)."""
    lens = np.asarray(lens, dtype=np.int64)
    k = len(lens)
    text = int(seq - lens.sum())
    if text < 0:
        raise ValueError("image tokens exceed the sequence length")
    cuts = np.sort(rng.integers(0, text + 1, size=k))
    gaps_before = np.diff(np.concatenate([[0], cuts]))
    starts = np.cumsum(gaps_before) + np.concatenate([[0], np.cumsum(lens)[:-1]])
    return starts.astype(np.int32)


def token_map_from_lens(rng: np.random.Generator, batch: int, seq: int, hidden: int,
                        lens_per_sample: Sequence[Sequence[int]]) -> TokenMap:
    samp, start, length = [], [], []
    for b in range(batch):
        lens = list(lens_per_sample[b])
        if not lens:
            continue
        st = place_spans(rng, seq, lens)
        samp += [b] * len(lens)
        start += st.tolist()
        length += lens
    return TokenMap(batch, seq, hidden, np.array(samp, np.int32),
                    np.array(start, np.int32), np.array(length, np.int32))


def _draw_until(rng: np.random.Generator, lo: int, hi: int, target_rows: int,
                max_images: int) -> List[int]:
    lens: List[int] = []
    while sum(lens) < target_rows and len(lens) < max_images:
        lens.append(int(rng.integers(lo, hi + 1)))
    return lens


def tiny(seed: int = BASE_SEED + 1) -> Workload:
    """Config 1: vision DP2,TP1 -> LLM TP2,CP1,DP1; batch 2, 256 text tokens plus
    4 images x 16 tokens per sample (fused length 320), hidden 64."""
    rng = np.random.default_rng(seed)
    tm = token_map_from_lens(rng, 2, 256 + 4 * 16, 64, [[16] * 4] * 2)
    return Workload("tiny", Grid(tp=1, dp=2), Grid(tp=2, cp=1, dp=1), [tm], seed)


def colocated4(seed: int = BASE_SEED + 2) -> Workload:
    """Config 2: vision TP1,DP4 -> LLM TP4,DP1 on the same four ranks; batch 4,
    8 images x 1024 tokens per sample plus 8192 text tokens (fused 16384),
    hidden 4096."""
    rng = np.random.default_rng(seed)
    tm = token_map_from_lens(rng, 4, 8192 + 8 * 1024, 4096, [[1024] * 8] * 4)
    return Workload("colocated4", Grid(tp=1, dp=4), Grid(tp=4, cp=1, dp=1), [tm], seed)


def shuffle_spans(rng: np.random.Generator, tm: TokenMap) -> TokenMap:
    """The same set of spans with, inside every sample, the spans handed to the
    images in a seeded random order: image k of a sample no longer sits before
    image k+1 in the sequence.  Source rows stay in image order, so the
    transform has to follow the token map, not the position order."""
    samp = np.asarray(tm.img_sample)
    start = np.asarray(tm.img_start).copy()
    length = np.asarray(tm.img_len).copy()
    for b in np.unique(samp):
        idx = np.flatnonzero(samp == b)
        perm = rng.permutation(len(idx))
        start[idx] = start[idx[perm]]
        length[idx] = length[idx[perm]]
    return replace(tm, img_start=start.astype(np.int32), img_len=length.astype(np.int32))


def split_edges(rng: np.random.Generator, tm: TokenMap, n_edges: int) -> List[TokenMap]:
    """Deals the spans of one token map out to n_edges encoders at random (a
    graph join: several encoders feed disjoint spans of the same sequence).
    Every returned map keeps the sample-major order; an edge may get no span."""
    owner = rng.integers(0, n_edges, size=tm.n_images)
    out = []
    for e in range(n_edges):
        sel = owner == e
        out.append(TokenMap(tm.batch, tm.seq, tm.hidden, tm.img_sample[sel], tm.img_start[sel],
                            tm.img_len[sel], None, tm.dtype))
    return out


def colocated4_dense(seed: int = BASE_SEED + 2) -> Workload:
    """Config 2 under its other reading: the stated sequence length of 8192 is
    the fused length, so the 8 images x 1024 tokens of a sample tile the whole
    sequence with no text between them; the images of a sample take the eight
    slots in a seeded random order."""
    rng = np.random.default_rng(seed)
    samp = np.repeat(np.arange(4), 8)
    start = np.concatenate([rng.permutation(8) * 1024 for _ in range(4)])
    tm = TokenMap(4, 8192, 4096, samp.astype(np.int32), start.astype(np.int32),
                  np.full(32, 1024, np.int32))
    return Workload("colocated4_dense", Grid(tp=1, dp=4), Grid(tp=4, cp=1, dp=1), [tm], seed)


def long_context(seed: int = BASE_SEED + 3, n_images: Optional[int] = None) -> Workload:
    """Config 3: vision DP8 -> LLM TP4,CP8 with the load-balanced split; one
    sample of 131072 fused tokens, hidden 5120; image lengths U{256..2304} drawn
    until they cover 30 % of the sequence (at most 32 images), or exactly
    n_images of them when given."""
    rng = np.random.default_rng(seed)
    seq = 131072
    if n_images is None:
        lens = _draw_until(rng, 256, 2304, int(0.30 * seq), 32)
    else:
        lens = [int(rng.integers(256, 2305)) for _ in range(n_images)]
    tm = token_map_from_lens(rng, 1, seq, 5120, [lens])
    return Workload("long_context", Grid(tp=1, dp=8),
                    Grid(tp=4, cp=8, dp=1, cp_split=CP_ZIGZAG), [tm], seed)


def non_colocated(seed: int = BASE_SEED + 4, n_microbatches: int = 16) -> Workload:
    """Config 4: vision DP4 on ranks 0-3 -> LLM TP2,CP2 on ranks 4-7; 16
    microbatches of one 16384-token sample, hidden 8192, 4-16 images of 576
    tokens each."""
    rng = np.random.default_rng(seed)
    maps = []
    for _ in range(n_microbatches):
        k = int(rng.integers(4, 17))
        maps.append(token_map_from_lens(rng, 1, 16384, 8192, [[576] * k]))
    return Workload("non_colocated", Grid(tp=1, dp=4, rank_offset=0),
                    Grid(tp=2, cp=2, dp=1, rank_offset=4, cp_split=CP_ZIGZAG), maps, seed)


def large_scale(seed: int = BASE_SEED + 5) -> Workload:
    """Config 5: vision TP2,DP16 -> LLM TP8,CP4,DP1, 32 ranks each side; one
    sample of 65536 fused tokens, hidden 12288, variable-resolution images of
    64-4096 tokens drawn until they cover half the sequence."""
    rng = np.random.default_rng(seed)
    seq = 65536
    lens = _draw_until(rng, 64, 4096, seq // 2, 1 << 30)
    if sum(lens) > seq:
        lens[-1] -= sum(lens) - seq
    tm = token_map_from_lens(rng, 1, seq, 12288, [lens])
    return Workload("large_scale", Grid(tp=2, dp=16),
                    Grid(tp=8, cp=4, dp=1, cp_split=CP_ZIGZAG), [tm], seed)


def scaled(w: Workload, hidden: int) -> Workload:
    """The same grids and spans at another hidden size (keeps every segment
    boundary of the full problem while shrinking the bytes)."""
    return replace(w, name=f"{w.name}_h{hidden}",
                   maps=[replace(m, hidden=hidden) for m in w.maps])


CONFIGS = {
    "tiny": tiny,
    "colocated4": colocated4,
    "colocated4_dense": colocated4_dense,
    "long_context": long_context,
    "non_colocated": non_colocated,
    "large_scale": large_scale,
}


def random_layout_case(rng: np.random.Generator, max_seq_units: int = 6):
    """A small random problem for brute-force tests: random grids, split rule,
    row order, explicit or default image placement, ragged spans."""
    tp_s = int(rng.choice([1, 2]))
    dp_s = int(rng.choice([1, 2, 3, 4, 8]))
    tp_d = int(rng.choice([1, 2, 3, 4]))
    cp_d = int(rng.choice([1, 2, 4]))
    dp_d = int(rng.choice([1, 2]))
    batch = dp_d * int(rng.choice([1, 2]))
    seq = 2 * cp_d * int(rng.integers(1, max_seq_units + 1)) * int(rng.choice([1, 3, 4]))
    hidden = int(rng.choice([8, 16, 24]))
    lens_per_sample = []
    for _ in range(batch):
        n = int(rng.integers(0, 5))
        lens, budget = [], seq
        for _ in range(n):
            if budget <= 0:
                break
            ln = int(rng.integers(1, max(2, min(budget, seq // 2 + 1))))
            ln = min(ln, budget)
            lens.append(ln)
            budget -= ln
        lens_per_sample.append(lens)
    tm = token_map_from_lens(rng, batch, seq, hidden, lens_per_sample)
    if tm.n_images and rng.random() < 0.5:
        # explicit, non-decreasing image -> source-dp assignment (ranks may be empty)
        tm.img_src_dp = np.sort(rng.integers(0, dp_s, size=tm.n_images)).astype(np.int32)
    src = Grid(tp=tp_s, dp=dp_s, rank_offset=int(rng.integers(0, 3)))
    dst = Grid(tp=tp_d, cp=cp_d, dp=dp_d, rank_offset=int(rng.integers(0, 9)),
               cp_split=int(rng.choice([CP_CONTIGUOUS, CP_ZIGZAG])),
               row_order=int(rng.choice([ROW_BSH, ROW_SBH])))
    return src, dst, tm


def random_wide_case(rng: np.random.Generator):
    """A medium-size random problem with wide grids (CP up to 16, destination TP
    up to 16, many images of very different lengths, up to 8 samples): more
    segments than one search-tree node holds, spans across many chunk borders."""
    while True:
        tp_s = int(rng.choice([1, 2, 4]))
        dp_s = int(rng.choice([1, 3, 8, 16, 32]))
        tp_d = int(rng.choice([1, 2, 5, 8, 16]))
        cp_d = int(rng.choice([1, 2, 4, 8, 16]))
        dp_d = int(rng.choice([1, 2, 4]))
        if tp_s * dp_s + tp_d * cp_d * dp_d <= 448:          # the library's buffer limit
            break
    batch = dp_d * int(rng.choice([1, 2]))
    seq = 2 * cp_d * tp_d * int(rng.integers(2, 40))
    hidden = int(rng.choice([8, 12, 64]))
    lens_per_sample = []
    for _ in range(batch):
        lens, budget = [], int(seq * rng.uniform(0.2, 1.0))
        while budget > 0 and len(lens) < 40:
            ln = min(budget, int(rng.choice([1, 2, 7, 33, 150, 700])))
            lens.append(ln)
            budget -= ln
        lens_per_sample.append(lens)
    tm = token_map_from_lens(rng, batch, seq, hidden, lens_per_sample)
    if rng.random() < 0.3:
        tm = shuffle_spans(rng, tm)
    if tm.n_images and rng.random() < 0.5:
        tm.img_src_dp = np.sort(rng.integers(0, dp_s, size=tm.n_images)).astype(np.int32)
    src = Grid(tp=tp_s, dp=dp_s)
    dst = Grid(tp=tp_d, cp=cp_d, dp=dp_d, cp_split=int(rng.choice([CP_CONTIGUOUS, CP_ZIGZAG])),
               row_order=int(rng.choice([ROW_BSH, ROW_SBH])),
               tp_mode=int(rng.choice([TP_REPLICATE, TP_SEQ_SHARD])))
    return src, dst, tm


def random_bf16(shape, seed: int, device: str = "cpu", scale: float = 1.0):
    """N(0, scale^2) drawn in fp32 by torch's seeded generator on `device`, then
    rounded to bf16 by torch.  Returns a torch.bfloat16 tensor on `device`."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    n = int(np.prod(shape))
    if n == 0:
        return torch.empty(tuple(shape), dtype=torch.bfloat16, device=device)
    if device == "cpu" and n > (1 << 26):
        # large host tensors: fill in slabs to bound the fp32 temporary
        out = torch.empty(n, dtype=torch.bfloat16)
        step = 1 << 24
        for i in range(0, n, step):
            m = min(step, n - i)
            out[i:i + m] = (torch.randn(m, generator=g, dtype=torch.float32) * scale).to(torch.bfloat16)
        return out.view(tuple(shape))
    x = torch.randn(tuple(shape), generator=g, dtype=torch.float32, device=device)
    if scale != 1.0:
        x = x * scale
    return x.to(torch.bfloat16)


def bf16_bits(t) -> np.ndarray:
    """Raw 16-bit patterns of a CPU bf16 tensor as a numpy uint16 array (shares
    memory with the tensor)."""
    import torch
    assert t.dtype == torch.bfloat16 and t.device.type == "cpu"
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def bits_to_bf16(a: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16)
