"""Host-side behaviour around the library: bench.py's refusal of more than one
GPU, and the binding's refusal to work without the built library (there is no
CPU or PyTorch path to fall back to)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_refuses_a_multi_rank_launch():
    env = dict(os.environ, WORLD_SIZE="2", RANK="0", LOCAL_RANK="0")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], env=env,
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_binding_raises_without_the_built_library(monkeypatch, tmp_path):
    from paper_2605_27678_amd import binding, workloads as wl
    monkeypatch.setattr(binding, "_handle", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libhp.so"))
    tm = wl.tiny().maps[0]
    with pytest.raises(RuntimeError, match="no CPU or PyTorch fallback"):
        binding.hp_plan_create_host(wl.Grid(dp=2), wl.Grid(tp=2), tm)
    with pytest.raises(RuntimeError, match="is missing"):
        binding.hp_version()


def test_product_package_does_not_import_the_oracle():
    """The oracle is test infrastructure: nothing under the package may import it."""
    pkg = os.path.join(ROOT, "paper_2605_27678_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".hpp", ".h")):
                for line in open(os.path.join(dirpath, f), encoding="utf-8"):
                    code = line.split("#")[0].split("//")[0]
                    if "import" in code or "include" in code or "CDLL" in code or "open(" in code:
                        assert "oracle" not in code.lower(), (os.path.join(dirpath, f), line)


@pytest.mark.parametrize("compiler,std", [("gcc", "-std=c99"), ("g++", "-std=c++11")])
def test_header_is_plain_c(compiler, std, tmp_path):
    """include/hp.h compiles on its own as strict C99 and as C++: no HIP or
    torch types cross the boundary."""
    src = tmp_path / ("t.c" if compiler == "gcc" else "t.cpp")
    src.write_text('#include "hp.h"\nint main(void) { hp_launch_t l; hp_plan_info_t i; (void)l; (void)i; '
                   'return sizeof(hp_layout_t) == 32 && HP_AUTO == -1 ? 0 : 1; }\n')
    exe = tmp_path / "t"
    r = subprocess.run([compiler, std, "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                        str(src), "-o", str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr
    assert subprocess.run([str(exe)], timeout=30).returncode == 0


def test_counter_traffic_is_quoted_only_for_the_sources_and_shapes_it_was_measured_with(tmp_path, monkeypatch):
    """bench.py's roofline.traffic comes from a committed rocprofv3 summary; it
    must turn into null as soon as the kernel sources or a launch shape differ
    from what the summary records."""
    sys.path.insert(0, ROOT)
    import bench
    monkeypatch.setattr(bench, "PROFILES", str(tmp_path))
    shapes = {"fwd": dict(tile_bytes=2048, block_threads=64, waves_per_cu=12, nontemporal=2),
              "bwd": dict(tile_bytes=1024, block_threads=64, waves_per_cu=16, nontemporal=3)}

    def write(digest, fwd="2048,64,12,2", bwd="1024,64,16,3"):
        (tmp_path / "hbm_traffic_long_context.txt").write_text(
            "# comment = ignored\nhead = abc1234\nkernel_sources_sha256 = %s\nshape_fwd = %s\nshape_bwd = %s\n"
            "forward_bytes_per_launch = 2055420910     # algorithmic 2055116800\nbackward_bytes_per_launch = 2055260453\n"
            "forward_bytes_per_boundary_byte = 5.0007\nbackward_bytes_per_boundary_byte = 5.0003\n" % (digest, fwd, bwd))

    assert bench.traffic_for("long_context", shapes, "hp_forward_kernel") == (None, None, None)     # no summary at all
    write(bench.kernel_source_digest())
    t, per, src = bench.traffic_for("long_context", shapes, "hp_forward_kernel")
    assert (t, per) == (2055420910.0, 5.0007) and src["matches_this_run"] and src["head"] == "abc1234"
    assert src["file"] == "profiles/hbm_traffic_long_context.txt" and src["shapes"]["fwd"] == "2048,64,12,2"
    t, per, _ = bench.traffic_for("long_context", shapes, "hp_backward_kernel")
    assert (t, per) == (2055260453.0, 5.0003)
    other = {"fwd": dict(shapes["fwd"], waves_per_cu=8), "bwd": shapes["bwd"]}                      # another launch shape
    t, per, src = bench.traffic_for("long_context", other, "hp_forward_kernel")
    assert t is None and per is None and src["matches_this_run"] is False
    write("0" * 64)                                                                                 # other kernel sources
    t, per, src = bench.traffic_for("long_context", shapes, "hp_forward_kernel")
    assert t is None and src["matches_this_run"] is False
    assert bench.traffic_label(dict(workload="long_context", accumulate=True)) == "long_context_accumulate"
    assert bench.traffic_label(dict(workload="large_scale", seq_shard=True, dtype="f32")) == "large_scale_seq_shard_f32"


def test_plain_c_client_links_against_the_library(tmp_path):
    """The boundary is a C ABI: a C99 program that includes only include/hp.h,
    compiled with gcc and linked against libhp.so, builds and reads a plan."""
    from paper_2605_27678_amd import binding
    exe = tmp_path / "abi_client"
    libdir = os.path.dirname(binding.LIB_PATH)
    rocm = "/opt/rocm/lib"
    r = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                        os.path.join(ROOT, "tests", "abi_client.c"), "-o", str(exe),
                        "-L", libdir, "-l:libhp.so", f"-Wl,-rpath,{libdir}", f"-Wl,-rpath-link,{rocm}", f"-Wl,-rpath,{rocm}"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "abi client ok" in r.stdout, r.stdout + r.stderr
