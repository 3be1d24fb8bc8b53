"""Host code under sanitizers (no GPU, no kernel): the library's host layer in a native program built with
AddressSanitizer + UndefinedBehaviorSanitizer, and the C oracle built with UndefinedBehaviorSanitizer."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2603_16104_amd", "csrc")


@pytest.mark.timeout(600)
def test_host_layer_under_asan_and_ubsan(tmp_path):
    if shutil.which("g++") is None or not os.path.exists("/opt/rocm/lib/libamdhip64.so"):
        pytest.skip("needs g++ and the HIP runtime library")
    exe = str(tmp_path / "host_check")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", os.path.join(ROOT, "tests", "native", "host_check.cpp"),
           os.path.join(CSRC, "api.cpp"), os.path.join(CSRC, "trt.cpp"), os.path.join(CSRC, "cache.cpp"),
           "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-o", exe]
    subprocess.check_call(cmd)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    out = r.stdout + r.stderr
    assert r.returncode == 0 and "0 failed checks" in out, out[-4000:]
    assert "AddressSanitizer" not in out and "runtime error" not in out and "LeakSanitizer" not in out, out[-4000:]


@pytest.mark.timeout(600)
def test_oracle_under_ubsan(tmp_path):
    if shutil.which("gcc") is None:
        pytest.skip("needs gcc")
    so = str(tmp_path / "liboracle_ubsan.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-fsanitize=undefined",
                           "-fno-sanitize-recover=undefined", "-o", so, os.path.join(ROOT, "oracle", "oracle.c"), "-lm"])
    code = f"""
import sys
sys.path.insert(0, {ROOT!r})
import numpy as np
from oracle import oracle as orc
orc._SO = {so!r}
orc.build = lambda force=False: orc._SO
from paper_2603_16104_amd import workloads as wl
pre, dec = wl.config1()
for w in (pre, dec, wl.random_forest_workload(7, kv_dtype=wl.KV_FP8_E4M3), wl.random_forest_workload(8, mode="prefill", src_dtype="fp32", kv_dtype=wl.KV_FP32)):
    hp = orc.HostPool(w.num_pages, w.num_kv_heads, w.kv_dtype)
    hp.fill_from(w)
    o, l = orc.run_workload(w, hp)
    assert np.isfinite(o).all()
    f = w.forest
    orc.flatten_tree(f.nodes, f.node_pages, f.req_leaf, max(1, f.max_pages_per_req()))
    orc.prefill_usage(f.nodes, f.req_leaf)
assert [orc.e4m3_encode(orc.e4m3_value(c)) for c in range(256) if (c & 0x7F) != 0x7F] == [c for c in range(256) if (c & 0x7F) != 0x7F]
print("oracle ok")
"""
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=500)
    out = r.stdout + r.stderr
    assert r.returncode == 0 and "oracle ok" in out and "runtime error" not in out, out[-4000:]
