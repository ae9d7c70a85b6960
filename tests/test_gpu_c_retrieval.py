"""Asynchronous retrieval driven from a plain C program (gcc, C99): the receive slots without any Python in
the loop, for one request per arrival and for several, on a small shape with every request checked and on
the burst workload's shape for the host cost per request."""
import os
import subprocess

import pytest

from paper_2408_08147_amd import kvx

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def build_c_retrieval(tmp_path):
    exe = tmp_path / "c_retrieval"
    libdir = os.path.dirname(kvx.lib_path())
    kvx.load()
    cmd = ["gcc", "-std=gnu99", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include",
           "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "c_retrieval.c"),
           "-L", libdir, "-lkvx", "-L", "/opt/rocm/lib", "-lamdhip64",
           "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib", "-o", str(exe)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    return exe


def test_c_retrieval_builds(tmp_path):
    build_c_retrieval(tmp_path)


@pytest.mark.gpu
def test_c_retrieval_small_every_request_checked(tmp_path):
    exe = build_c_retrieval(tmp_path)
    res = subprocess.run([str(exe), "24", "3", "2", "64", "2", "16", "1,3", "1,5", "1"],
                         capture_output=True, text=True, timeout=120)
    print(res.stdout)
    assert res.returncode == 0, (res.stdout[-2000:], res.stderr[-2000:])
    assert "retrieval ok: 192 rows checked" in res.stdout


@pytest.mark.gpu
@pytest.mark.timeout(400)
def test_c_retrieval_burst_shape(tmp_path):
    """512 requests of the burst workload's shape; prints the microseconds per request from C."""
    exe = build_c_retrieval(tmp_path)
    res = subprocess.run([str(exe), "512", "40", "8", "128", "1", "16", "1,2,4", "1,4,16", "16"],
                         capture_output=True, text=True, timeout=380)
    print(res.stdout)
    assert res.returncode == 0, (res.stdout[-2000:], res.stderr[-2000:])
    assert "retrieval ok" in res.stdout and res.stdout.count("us per request") == 9
