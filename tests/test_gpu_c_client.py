"""A C program drives the library on the GPU without Python in between and
compares with the CPU oracle's results stored in tests/golden/tiny_case.bin
(written by tests/golden/make_tiny_case.py, which calls only the oracle)."""
import os
import shutil
import subprocess

import numpy as np
import pytest

import oracle
import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CASE = os.path.join(ROOT, "tests", "golden", "tiny_case.bin")


def test_stored_case_is_what_the_oracle_computes_now():
    """The stored file holds the oracle's current results for the Tiny set (so a
    change of the oracle or of the input recipe cannot go unnoticed)."""
    ws = workloads.make_weight_set("tiny")
    rb = workloads.config_bytes("tiny")
    stream = oracle.pack(ws.weights, ws.layer_offsets, rb)
    blob = open(CASE, "rb").read()
    assert blob[:4] == b"ADTT"
    assert ws.weights.astype("<f4").tobytes() in blob
    assert stream.tobytes() in blob
    assert oracle.unpack(stream, ws.layer_offsets, rb).astype("<f4").tobytes() in blob
    assert oracle.stats(ws.weights, ws.layer_offsets).astype("<f8").tobytes() == blob[-72:]
    assert stream.size == 35168 and np.array_equal(rb, [2, 3, 4])


@pytest.mark.gpu
def test_c_program_packs_unpacks_and_takes_statistics_on_the_gpu(tmp_path):
    import paper_2004_02297_amd as adt
    adt.load_library()
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    lib = adt.lib_path()
    exe = tmp_path / "gpu_client"
    subprocess.check_call(["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-Werror",
                           "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"),
                           "-I", "/opt/rocm/include",
                           os.path.join(ROOT, "tests", "c_client", "gpu_client.c"), "-o", str(exe),
                           lib, "-L/opt/rocm/lib", "-lamdhip64", "-lm",
                           "-Wl,-rpath," + os.path.dirname(lib), "-Wl,-rpath,/opt/rocm/lib"])
    out = subprocess.run([str(exe), CASE], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0 and "c client ok: 3 layers, 10160 weights, 35168 stream bytes" in out.stdout, \
        (out.returncode, out.stdout, out.stderr)
