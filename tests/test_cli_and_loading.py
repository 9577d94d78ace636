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
