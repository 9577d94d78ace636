"""The CPU oracle built with AddressSanitizer + UBSan (no GPU): the hand-worked
example and random small layouts (both TP modes, both split rules, both row
orders, empty source ranks) run through a C driver that allocates every buffer
at its exact size; no sanitizer report, and the results equal the fixture and the
ordinary build's."""
import json
import os
import subprocess

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2605_27678_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(ROOT, "tests", "golden")


def _bits(vals):
    return wl.bf16_bits(torch.tensor(vals, dtype=torch.float32).to(torch.bfloat16)).copy()


def _grid_words(g):
    return [g.tp, g.cp, g.dp, g.tp_mode, g.cp_split, g.row_order]


def _build(tmp_path):
    exe = tmp_path / "oracle_sanitized"

    def build(sanitizers):
        r = subprocess.run(["gcc", "-std=c11", "-O1", "-g", *sanitizers, "-fno-sanitize-recover=all", "-fopenmp",
                            "-fno-fast-math", "-ffp-contract=off", "-Wall", "-Wextra",
                            os.path.join(ROOT, "tests", "oracle_sanitized.c"), os.path.join(ROOT, "oracle", "hp_oracle.c"),
                            "-o", str(exe)], capture_output=True, text=True, timeout=300)
        assert r.returncode == 0, r.stderr

    build(["-fsanitize=address,undefined", "-static-libasan"])
    probe_in, probe_out = tmp_path / "probe.in", tmp_path / "probe.out"
    probe_in.write_bytes(np.zeros(1, np.int32).tobytes())
    first = subprocess.run([str(exe), str(probe_in), str(probe_out)], capture_output=True, text=True, timeout=120)
    if first.returncode != 0 and "ASan runtime does not come first" in first.stderr:
        build(["-fsanitize=undefined"])              # another library is preloaded here: UBSan only
    return exe


def test_oracle_under_sanitizers(tmp_path):
    exe = _build(tmp_path)
    rng = np.random.default_rng(31)
    cases = []
    # the hand-worked example (hidden 1)
    g = json.load(open(os.path.join(GOLDEN, "worked_example_zigzag.json")))
    mk = lambda d: wl.Grid(tp=d.get("tp", 1), cp=d.get("cp", 1), dp=d.get("dp", 1),
                           cp_split=wl.CP_ZIGZAG if d.get("cp_split") == "zigzag" else wl.CP_CONTIGUOUS,
                           row_order=wl.ROW_SBH if d.get("row_order") == "sbh" else wl.ROW_BSH)
    src, dst = mk(g["src"]), mk(g["dst"])
    tm = wl.TokenMap(g["batch"], g["seq"], g["hidden"], g["img_sample"], g["img_start"], g["img_len"])
    prob = oracle.Problem(src, dst, tm)
    cases.append((src, dst, tm, [_bits(b).reshape(-1, 1) for b in g["src_bufs"]],
                  [_bits([g["dst_text"]] * prob.dst_rows()).reshape(-1, 1) for _ in range(prob.n_dst)],
                  [_bits(g["dst_grads"][str(j)]).reshape(-1, 1) for j in range(prob.n_dst)]))
    from dataclasses import replace
    while len(cases) < 25:
        src, dst, tm = wl.random_layout_case(rng)
        if len(cases) % 3 == 0:
            if (tm.seq // dst.cp) % dst.tp:
                continue
            dst = replace(dst, tp_mode=wl.TP_SEQ_SHARD)
        prob = oracle.Problem(src, dst, tm)
        rnd = lambda rows: rng.integers(0, 0x7F00, size=(rows, tm.hidden), dtype=np.uint16)   # finite bf16 patterns
        cases.append((src, dst, tm, [rnd(r) for r in prob.src_rows()],
                      [rnd(prob.dst_rows()) for _ in range(prob.n_dst)], [rnd(prob.dst_rows()) for _ in range(prob.n_dst)]))
    blob = [np.array([len(cases)], np.int32).tobytes()]
    for src, dst, tm, sb, db, gb in cases:
        blob.append(np.array(_grid_words(src) + _grid_words(dst) +
                             [tm.batch, tm.seq, tm.hidden, tm.n_images, int(tm.img_src_dp is not None)], np.int32).tobytes())
        for a in (tm.img_sample, tm.img_start, tm.img_len):
            blob.append(np.ascontiguousarray(a, np.int32).tobytes())
        if tm.img_src_dp is not None:
            blob.append(np.ascontiguousarray(tm.img_src_dp, np.int32).tobytes())
        for a in sb + db + gb:
            blob.append(np.ascontiguousarray(a, np.uint16).tobytes())
    fin, fout = tmp_path / "cases.in", tmp_path / "cases.out"
    fin.write_bytes(b"".join(blob))
    r = subprocess.run([str(exe), str(fin), str(fout)], capture_output=True, text=True, timeout=300,
                       env=dict(os.environ, OMP_NUM_THREADS="2"))
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.split() == ["cases", str(len(cases))]
    raw = fout.read_bytes()
    pos = 0

    def take(dtype, shape):
        nonlocal pos
        n = int(np.prod(shape)) * np.dtype(dtype).itemsize
        a = np.frombuffer(raw, dtype, count=int(np.prod(shape)), offset=pos).reshape(shape)
        pos += n
        return a

    for ci, (src, dst, tm, sb, db, gb) in enumerate(cases):
        prob = oracle.Problem(src, dst, tm)
        H, dr, sr = tm.hidden, prob.dst_rows(), prob.src_rows()
        got_dst = [take(np.uint16, (dr, H)) for _ in range(prob.n_dst)]
        got_sg = [take(np.uint16, (r, H)) for r in sr]
        got_sg2 = [take(np.uint16, (r, H)) for r in sr]
        got_acc = [take(np.float32, (r, H)) for r in sr]
        fm_buf, fm_row = take(np.int32, (dr,)), take(np.int64, (dr,))
        if ci == 0:                                   # against the fixture's hand-derived values
            for j in range(prob.n_dst):
                assert got_dst[j].ravel().tolist() == _bits(g["dst_expected"][str(j)]).tolist()
            for i, exp in enumerate(g["src_grads_expected"]):
                assert got_sg[i].ravel().tolist() == _bits(exp).tolist()
        want_dst = [a.copy() for a in db]
        prob.forward(sb, want_dst)
        want_sg = [np.full((r, H), 0xEEEE, np.uint16) for r in sr]
        prob.backward_bf16(gb, want_sg)
        want_acc = [np.zeros((r, H), np.float32) for r in sr]
        prob.backward_accumulate(gb, want_acc)
        wb, wr = prob.forward_map(0)
        assert all(np.array_equal(a, b) for a, b in zip(got_dst, want_dst)), ci
        assert all(np.array_equal(a, b) for a, b in zip(got_sg, want_sg)), ci
        assert all(np.array_equal(a, b) for a, b in zip(got_sg2, want_sg)), ci
        assert all(np.array_equal(a.view(np.uint32), b.view(np.uint32)) for a, b in zip(got_acc, want_acc)), ci
        assert np.array_equal(fm_buf, wb) and np.array_equal(fm_row, wr), ci
    assert pos == len(raw)
