"""Host-side checks of what the repository promises around the library: the benchmark refuses
more than one GPU, the product package never reaches into the oracle (or any scratch folder),
and the sources carry the compile flag the build needs."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_product_package_does_not_import_the_oracle_or_scratch_files():
    pkg = os.path.join(ROOT, "paper_2503_08640_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".hpp")):
                text = open(os.path.join(dirpath, f), encoding="utf-8").read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), f
                assert not re.search(r"[\"'/]_work/", text) and "/root/reference" not in text, f


def test_every_hip_source_is_built_with_packed_fp32_ops_disabled():
    text = open(os.path.join(ROOT, "paper_2503_08640_amd", "build.py"), encoding="utf-8").read()
    assert "-packed-fp32-ops" in text and "--offload-arch=gfx950" in text
    csrc = os.path.join(ROOT, "paper_2503_08640_amd", "csrc")
    listed = set(re.findall(r'"([a-z_0-9]+\.(?:hip|cpp))"', text))
    present = {f for f in os.listdir(csrc) if f.endswith((".hip", ".cpp"))}
    assert present <= listed, present - listed
    for f in present:
        assert "v_pk_fma_f32" not in open(os.path.join(csrc, f), encoding="utf-8").read()
