"""Mutation audit of the CPU oracle's pins (no GPU).

Each case plants ONE plausible mistake in a scratch copy of oracle/hp_oracle.c
(never in place), builds that copy and runs the oracle's pins
(tests/test_oracle_pins.py) against it in a subprocess.  The audit passes when
every planted mistake makes at least one pin fail: a mistake the pins cannot see
would mean that part of the oracle is pinned by nothing but itself.

The scratch tree holds copies of oracle/, of the pin file and its fixtures, and
a link to the input generators; the subprocess runs inside it, so `import oracle`
resolves to the mutated copy.
"""
import concurrent.futures
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# (name, text to find exactly once in hp_oracle.c, replacement)
MUTANTS = [
    # --- destination walk ---------------------------------------------------
    ("zigzag second half keeps no chunk offset",
     "(2 * (int64_t)dst->cp - 1 - cp) * c + (s_l - c)", "(2 * (int64_t)dst->cp - 1 - cp) * c + (s_l)"),
    ("zigzag mirror chunk off by one",
     "(2 * (int64_t)dst->cp - 1 - cp) * c + (s_l - c)", "(2 * (int64_t)dst->cp - cp) * c + (s_l - c)"),
    ("zigzag first half uses the contiguous stride",
     "if (s_l < c) s = (int64_t)cp * c + s_l;", "if (s_l < c) s = (int64_t)cp * scp + s_l;"),
    ("tp is the slowest digit of the buffer index",
     "int32_t tp = buf % dst->tp;", "int32_t tp = buf / (dst->cp * dst->dp);"),
    ("cp and dp digits swapped",
     "int32_t cp = (buf / dst->tp) % dst->cp;", "int32_t cp = (buf / dst->tp) / dst->dp;"),
    ("[S,B,H] decoded as [B,S,H]",
     "else                     { s_l = row / bl_n; b_l = row % bl_n; }",
     "else                     { s_l = row % sl_n; b_l = row / sl_n; }"),
    ("sequence-sharded piece offset dropped",
     "s_l += (int64_t)tp * sl_n;", "s_l += 0;"),
    ("destination dp rank ignored",
     "*b_out = (int32_t)(dp * bl_n + b_l);", "*b_out = (int32_t)(b_l);"),
    ("contiguous split uses the zigzag chunk",
     "s = (int64_t)cp * scp + s_l;", "s = (int64_t)cp * (scp / 2) + s_l;"),
    # --- image lookup and source side -----------------------------------------
    ("token index counted from the end of the image",
     "*j_out = (int32_t)(s - m->img_start[k]);", "*j_out = (int32_t)(m->img_start[k] + m->img_len[k] - 1 - s);"),
    ("span end inclusive",
     "s < (int64_t)m->img_start[k] + m->img_len[k]", "s <= (int64_t)m->img_start[k] + m->img_len[k]"),
    ("source offset counts images of lower ranks too",
     "if (orc_image_src_dp(src, m, e) == d)\n            off += m->img_len[e];",
     "if (orc_image_src_dp(src, m, e) <= d)\n            off += m->img_len[e];"),
    ("balanced intervals rounded up",
     "int64_t hi = ((int64_t)(d + 1) * K) / src->dp;", "int64_t hi = ((int64_t)(d + 1) * K + src->dp - 1) / src->dp;"),
    ("forward reads source copy dp instead of copy tp=0 of rank dp",
     "(const char *)src_bufs[d * src->tp + 0]", "(const char *)src_bufs[d + 0]"),
    ("forward map reports a non-leader copy",
     "src_buf[r] = d * src->tp;", "src_buf[r] = d * src->tp + (src->tp - 1);"),
    # --- bf16 rounding ------------------------------------------------------
    ("ties round up instead of to even",
     "if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u)))", "if (lower >= 0x8000u)"),
    ("truncation instead of rounding",
     "if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u)))", "if (0)"),
    ("NaN not forced quiet (payload in the low bits rounds to infinity)",
     "return (uint16_t)((u >> 16) | 0x0040u);", "return (uint16_t)(u >> 16);"),
    ("NaN test misses the discarded bits",
     "if ((u & 0x7fffffffu) > 0x7f800000u)", "if ((u & 0x7fff0000u) > 0x7f800000u)"),
    # --- orc_backward_bf16 ----------------------------------------------------
    ("bf16 backward: fold in descending tp",
     "for (int32_t t = 1; t < n_rep; ++t) {", "for (int32_t t = n_rep - 1; t >= 1; --t) {"),
    ("bf16 backward: subtract instead of add",
     "                acc = acc + g;\n            }\n            uint16_t out", "                acc = acc - g;\n            }\n            uint16_t out"),
    ("bf16 backward: only source copy 0 written",
     "src_grads[d * src->tp + ts][srow * H + h] = out;", "src_grads[d * src->tp + 0][srow * H + h] = out;"),
    ("bf16 backward: sequence-sharded TP buffers summed as if replicated",
     "const int32_t n_rep = dst->tp_mode == 1 ? 1 : dst->tp;   /* copies of each row */",
     "const int32_t n_rep = dst->tp;   /* copies of each row */"),
    ("bf16 backward: replicas not summed (leader's copy returned)",
     "const int32_t n_rep = dst->tp_mode == 1 ? 1 : dst->tp;   /* copies of each row */\n    const int32_t n_slices = n_dst / n_rep;",
     "const int32_t n_rep = 1;   /* copies of each row */\n    const int32_t n_slices = n_dst / (dst->tp_mode == 1 ? 1 : dst->tp);"),
    ("bf16 backward: fold rounded to bf16 after every add",
     "                acc = acc + g;\n            }\n            uint16_t out",
     "                acc = bf16_to_f32(f32_to_bf16(acc + g));\n            }\n            uint16_t out"),
    # --- orc_backward (binary32 / accumulate) ---------------------------------
    ("generic backward: sequence-sharded TP buffers summed as if replicated",
     "const int32_t n_rep = dst->tp_mode == 1 ? 1 : dst->tp;\n", "const int32_t n_rep = dst->tp;\n"),
    ("generic backward: fold restarts at every copy",
     "else acc = acc + g;", "else acc = g + 0 * acc;"),
    ("generic backward: last of three or more copies dropped",
     "for (int32_t t = 0; t < n_rep; ++t) {", "for (int32_t t = 0; t < n_rep - (n_rep > 2); ++t) {"),
    ("generic backward: fold starts from +0.0 (loses the sign of -0)",
     "if (t == 0) acc = g;          /* the fold starts AT copy 0, not at +0.0 */", "acc = acc + g; if (0) acc = g;"),
    ("generic backward: only source copy 0 written",
     "void *out = src_out[d * src->tp + ts];", "void *out = src_out[d * src->tp + 0];"),
    ("accumulate overwrites",
     "a = a + acc;", "a = acc + 0 * a;"),
    ("accumulate subtracts",
     "a = a + acc;", "a = a - acc;"),
    ("binary32 output rounded to bf16",
     "((float *)out)[srow * H + h] = acc;", "((float *)out)[srow * H + h] = bf16_to_f32(f32_to_bf16(acc));"),
    # --- orc_zero_image_rows ----------------------------------------------------
    ("zero rows: text rows blanked instead of image rows",
     "if (find_image(m, b, s, &k, &j))\n                memset(", "if (!find_image(m, b, s, &k, &j))\n                memset("),
    ("zero rows: only every TP-th buffer visited",
     "for (int32_t buf = 0; buf < n_dst; ++buf)\n        for (int64_t r = 0; r < rows; ++r) {\n            int32_t b, k, j; int64_t s;",
     "for (int32_t buf = 0; buf < n_dst; buf += dst->tp)\n        for (int64_t r = 0; r < rows; ++r) {\n            int32_t b, k, j; int64_t s;"),
    ("zero rows: half of every row",
     "memset((char *)dst_bufs[buf] + (size_t)r * row_bytes, 0, row_bytes);",
     "memset((char *)dst_bufs[buf] + (size_t)r * row_bytes, 0, row_bytes / 2);"),
    ("generic backward: descending fold",
     "float g = dtype == 0 ? bf16_to_f32(((const uint16_t *)dst_grads[buf0 + t])[r * H + h])\n"
     "                                     : ((const float *)dst_grads[buf0 + t])[r * H + h];",
     "float g = dtype == 0 ? bf16_to_f32(((const uint16_t *)dst_grads[buf0 + n_rep - 1 - t])[r * H + h])\n"
     "                                     : ((const float *)dst_grads[buf0 + n_rep - 1 - t])[r * H + h];"),
]


def _scratch_tree(tmp, idx, old, new):
    d = os.path.join(tmp, f"m{idx:02d}")
    os.makedirs(os.path.join(d, "oracle"))
    os.makedirs(os.path.join(d, "tests"))
    src = open(os.path.join(ROOT, "oracle", "hp_oracle.c")).read()
    assert src.count(old) == 1, f"mutant {idx}: the text to replace occurs {src.count(old)} times"
    open(os.path.join(d, "oracle", "hp_oracle.c"), "w").write(src.replace(old, new))
    for f in ("oracle.py", "__init__.py"):
        shutil.copy(os.path.join(ROOT, "oracle", f), os.path.join(d, "oracle", f))
    shutil.copy(os.path.join(ROOT, "tests", "test_oracle_pins.py"), os.path.join(d, "tests"))
    shutil.copy(os.path.join(ROOT, "tests", "conftest.py"), os.path.join(d, "tests"))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(d, "tests", "golden"))
    os.symlink(os.path.join(ROOT, "paper_2605_27678_amd"), os.path.join(d, "paper_2605_27678_amd"))
    # the mutated source must still compile (with the oracle's own build line): a
    # build error would fail every pin and prove nothing
    subprocess.run([sys.executable, "-c", "from oracle import oracle; oracle.build(force=True)"],
                   cwd=d, env=dict(os.environ, PYTHONPATH=d), check=True, capture_output=True, timeout=120)
    return d


def _run_pins(d):
    env = dict(os.environ, PYTHONPATH=d, OMP_NUM_THREADS="2", PYTHONDONTWRITEBYTECODE="1")
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(d, "tests", "test_oracle_pins.py"),
                          "-x", "-q", "-p", "no:cacheprovider"],
                         cwd=d, env=env, capture_output=True, text=True, timeout=600)
    return res.returncode, (res.stdout + res.stderr)[-1500:]


@pytest.fixture(scope="module")
def audit(tmp_path_factory):
    tmp = str(tmp_path_factory.mktemp("mutants"))
    # the unmodified copy first: the scratch set-up itself must be green
    clean = _scratch_tree(tmp, 99, "TEST INFRASTRUCTURE ONLY", "TEST INFRASTRUCTURE ONLY")
    trees = [_scratch_tree(tmp, i, old, new) for i, (_, old, new) in enumerate(MUTANTS)]
    with concurrent.futures.ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(_run_pins, [clean] + trees))
    return {"clean": results[0], "mutants": results[1:]}


def test_unmodified_copy_passes_every_pin(audit):
    rc, tail = audit["clean"]
    assert rc == 0, tail


@pytest.mark.parametrize("idx", range(len(MUTANTS)), ids=[m[0] for m in MUTANTS])
def test_planted_mistake_fails_a_pin(audit, idx):
    rc, tail = audit["mutants"][idx]
    # pytest's exit status 1 = tests were collected and run, and at least one failed
    assert rc != 0, f"mutant '{MUTANTS[idx][0]}' passes every pin\n{tail}"
    assert rc == 1, f"pins did not run for mutant '{MUTANTS[idx][0]}' (exit status {rc})\n{tail}"
