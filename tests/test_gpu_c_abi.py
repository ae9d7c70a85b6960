"""The C ABI from a plain C program (gcc, C99): plan, pack, unpack, host-side check of every row."""
import os
import subprocess

import pytest

from paper_2408_08147_amd import kvx

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def build_c_caller(tmp_path):
    exe = tmp_path / "c_abi_roundtrip"
    libdir = os.path.dirname(kvx.lib_path())
    kvx.load()
    cmd = ["gcc", "-std=gnu99", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include",
           "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "c_abi_roundtrip.c"),
           "-L", libdir, "-lkvx", "-L", "/opt/rocm/lib", "-lamdhip64",
           "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib", "-o", str(exe)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    return exe


def test_c_caller_builds(tmp_path):
    build_c_caller(tmp_path)


@pytest.mark.gpu
def test_c_caller_round_trip(tmp_path):
    exe = build_c_caller(tmp_path)
    res = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    print(res.stdout)
    assert res.returncode == 0, (res.stdout[-2000:], res.stderr[-2000:])
    assert "C ABI round trip ok" in res.stdout
